// Layouts of the per-chunk arrays that the chunk-flow kernel hands to the scan kernel.
//
// They are stored tile by tile in the register layout of the 16x16x32 bf16 MFMA, so that the
// consumer's load "one operand tile for one wavefront" is a single contiguous 1 KiB read
// instead of sixteen 16-byte pieces from sixteen different rows.  "lane" below is the lane id
// within the wavefront, r16 = lane & 15, g = lane >> 4; the 8 elements of a lane are indexed
// by e, and the contraction index of a 32-wide k-step is relabelled as
//     kk(g, e) = 4 g + e           for e < 4
//              = 16 + 4 g + e - 4  for e >= 4
// (two stacked accumulator tiles, see pf_common.cuh).
//
// With n = chunk * r virtual tokens and per chunk MT = n / 16, NKT = n / 32, CT = chunk / 16:
//
//   Tt [MT][NKT][64 lanes][8]   T[16 mt + r16][32 kt + kk(g, e)],  T = (Id + G)^{-1}   (A operand)
//                               only tiles with 2 kt <= mt exist (T is lower block-triangular);
//                               the others are neither written nor read
//   Pt [CT][NKT][64 lanes][8]   P[16 tt + r16][32 kt + kk(g, e)],  P = Mbar (.) Q K^T  (B operand of P^T)
//                               only tiles with 32 kt < r (16 tt + 16) exist (readout mask)
//
// Chunks are laid out one after another in (b, h, chunk) order: n * n elements of Tt and
// chunk * n elements of Pt per chunk.
#pragma once
