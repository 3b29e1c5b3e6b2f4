// Layouts of the library-owned KV caches: where element (token, head element) of a 32-token block lives.
// Host- and device-callable, no HIP header needed (the CPU tests compile it as it is).
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "attn_plan.h"

namespace bass {

// ---------------------------------------------------------------------------------------
// bf16 cache layout (library-owned).  A cache is [B][Hkv][nblk] blocks of 32 tokens; a block
// holds 32*D bf16 stored in the order the matrix cores consume them, so that a wavefront
// reads 1 KiB per load instruction (lane l reads bytes [16 l, 16 l + 16)) straight into an
// MFMA operand.
//   K block: [tile tt (2)][k-step t (D/32)][lane (64)][j (8)]
//            lane = grp*16 + r holds token 16*tt + r, head elements d = 32*t + 8*grp + j
//   V block: [d-tile mt (D/16)][lane (64)][j (8)]
//            lane = grp*16 + dr holds head element d = 16*mt + dr of the eight tokens
//            (j < 4: 4*grp + j ; j >= 4: 16 + 4*grp + (j-4))
// The V token order is the order in which the score tile leaves the QK^T MFMA, which is why
// the probabilities need no shuffle before the PV MFMA.
// ---------------------------------------------------------------------------------------
BASS_HD inline size_t k_elem_offset(int D, int tok_in_blk, int d) {
  const int tt = tok_in_blk >> 4, r = tok_in_blk & 15;
  const int t = d >> 5, grp = (d & 31) >> 3, j = d & 7;
  return (size_t)(((tt * (D >> 5) + t) * 64 + grp * 16 + r) * 8 + j);
}

BASS_HD inline size_t v_elem_offset(int /*D*/, int tok_in_blk, int d) {
  const int half = tok_in_blk >> 4, w = tok_in_blk & 15;
  const int grp = w >> 2, j = half * 4 + (w & 3);
  const int mt = d >> 4, dr = d & 15;
  return (size_t)((mt * 64 + grp * 16 + dr) * 8 + j);
}

// ---------------------------------------------------------------------------------------
// INT8 cache layout (BASS_DTYPE_INT8KV).  Same blocks of 32 tokens; a block holds the 32*D codes as
// 16-byte chunks per lane, so that a wavefront still reads 1 KiB per load instruction, followed by the
// block's 32 fp32 scales in token order (one per token of this kv head).
//   K block: [tile tt (2)][k-step ks (D/64)][lane (64)][j (16)] -- the operand order of the INT8 matrix
//            instruction (16x16x64): lane = grp*16 + r holds token 16*tt + r, head elements 64*ks + 16*grp + j
//   V block: the element order of the bf16 V layout above, fragment mt of a lane being 8 codes = 8 bytes,
//            two consecutive fragments per chunk: byte ((mt/2)*64 + lane)*16 + (mt%2)*8 + j
// ---------------------------------------------------------------------------------------
BASS_HD inline size_t i8_block_bytes(int D) { return (size_t)kBlockTokens * D + kBlockTokens * 4; }

BASS_HD inline size_t i8_k_offset(int D, int tok_in_blk, int d) {
  const int tt = tok_in_blk >> 4, r = tok_in_blk & 15;
  const int ks = d >> 6, grp = (d & 63) >> 4, j = d & 15;
  return (size_t)(((tt * (D >> 6) + ks) * 64 + grp * 16 + r) * 16 + j);
}

BASS_HD inline size_t i8_v_offset(int /*D*/, int tok_in_blk, int d) {
  const int half = tok_in_blk >> 4, w = tok_in_blk & 15;
  const int grp = w >> 2, j = half * 4 + (w & 3);
  const int f = d >> 4, lane = grp * 16 + (d & 15);
  return (size_t)(((f >> 1) * 64 + lane) * 16 + (f & 1) * 8 + j);
}

}  // namespace bass
