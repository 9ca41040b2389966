// Layouts of the per-chunk arrays that the chunk-flow kernel hands to the scan kernel.
//
// They are stored tile by tile in the register layout of the 16x16x32 bf16 MFMA, so that the
// consumer's load "one operand tile for one wavefront" is a single contiguous 1 KiB (or 512 B)
// read instead of sixteen 16-byte pieces from sixteen different rows.  "lane" below is the
// lane id within the wavefront, r16 = lane & 15, g = lane >> 4.
//
// With n = chunk * r virtual tokens, d = d_k = d_v, and per chunk
//   MT = n / 16, NKT = n / 32, DT = d / 16, NKS = d / 32, CT = chunk / 16:
//
//   Wt [MT][NKS][64 lanes][8]   -W[16 mt + r16][32 ks + 8 g + e]                (A operand)
//   Ut [MT][DT ][64 lanes][4]   U'[16 mt + 4 g + e][16 dt + r16]                (accumulator)
//   Kt [DT][NKT][64 lanes][8]   K[32 kt + 8 g + e][16 a + r16]                  (A operand of K^T)
//   Pt [CT][NKT][64 lanes][8]   P[16 tt + r16][32 kt + 4 g + e]       for e < 4 (B operand of P^T,
//                               P[16 tt + r16][32 kt + 16 + 4 g + e-4] for e >= 4  k relabelled)
//                               tiles with 32 kt >= r (16 tt + 16) are all zero and are neither
//                               written nor read
//   Qt [CT][NKS][64 lanes][8]   Q[16 tt + r16][32 ks + 8 g + e]                 (B operand of Q^T)
//
// Chunks are laid out one after another in (b, h, chunk) order.
#pragma once
#include <stddef.h>

namespace pf {

struct TileDims {
    int MT, NKT, DT, NKS, CT;
};
inline TileDims tile_dims(int d, int n, int chunk)
{
    return TileDims{n / 16, n / 32, d / 16, d / 32, chunk / 16};
}

}  // namespace pf
