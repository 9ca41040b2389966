// Index maps of the per-block operand-tile arrays: T = (Id + G)^{-1} and P = Mbar (.) Q K^T of
// Theorem 3.2 (ParallelFlow, arXiv 2504.00492) as the kernels hand them on.
//
// Every array is a sequence of 1 KiB tiles in the register layout of the 16x16x32 bf16 MFMA, so
// that "one operand tile for one wavefront" is a single contiguous, bank-conflict-free read.
// "lane" is the lane id within the wavefront, r16 = lane & 15, g = lane >> 4; the 8 elements of a
// lane are indexed by e, and the contraction index of a 32-wide k-step is relabelled as
//     kk(g, e) = 4 g + e           for e < 4
//              = 16 + 4 g + e - 4  for e >= 4
// (two stacked accumulator tiles, see pf_common.h).  With n = block * r virtual tokens per flow
// block, MT = n / 16, NKT = n / 32, CT = block / 16, NB = n / 32:
//
//   T tile (mt, kt)      [64 lanes][8]  T[16 mt + r16][32 kt + kk(g, e)]        (A operand)
//                        exists for 2 kt <= mt (T is lower block-triangular)
//   P tile (tt, kt)      [64 lanes][8]  P[16 tt + r16][32 kt + kk(g, e)]        (B operand of P^T)
//                        exists for 32 kt < r (16 tt + 16) (readout mask, inclusive in time)
//   -G^T tile (j, mi, i) [64 lanes][8]  -G[32 i + kk(g, e)][32 j + 16 mi + r16] (A operand), i > j
//   T_jj^T tile (j, mi)  [64 lanes][8]  T[32 j + kk(g, e)][32 j + 16 mi + r16]  (A operand)
//
// In global memory (split entry points) T and P use the full grids [MT][NKT] and [CT][NKT], n * n
// and block * n elements per block, blocks in (b, h, block) order; tiles that do not exist are
// neither written nor read.  In LDS (fused kernel) only existing tiles are stored, at the compact
// indices below.
#pragma once

namespace pf {

// Global memory, full grids: element offset of tile (rt, kt) inside its block's array, NKT
// k-steps per row of tiles (rt = mt for T, tt for P); lane l's eight elements follow at 8 l.
constexpr size_t full_tile_offset(int NKT, int rt, int kt) { return ((size_t)rt * NKT + kt) * 64 * 8; }

// T: row tile mt has mt / 2 + 1 tiles
constexpr int t_tile_index(int mt, int kt)
{
    const int a = mt >> 1;
    return ((mt & 1) ? (a + 1) * (a + 1) : a * (a + 1)) + kt;
}
constexpr int t_tile_count(int MT) { return t_tile_index(MT, 0); }

// P: k-steps (32 virtual tokens each) that the 16 tokens of tile tt see
constexpr int p_ksteps(int r, int tt) { return (r * (16 * tt + 16) + 31) / 32; }
constexpr int p_tile_index(int r, int tt, int kt)
{
    int s = 0;
    for (int i = 0; i < tt; ++i) s += p_ksteps(r, i);
    return s + kt;
}
constexpr int p_tile_count(int r, int CT) { return p_tile_index(r, CT, 0); }

// -G^T: block-column j has two row halves (mi) of NB - 1 - j tiles each
constexpr int g_tile_index(int NB, int j, int mi, int i)
{
    int s = 0;
    for (int q = 0; q < j; ++q) s += 2 * (NB - 1 - q);
    return s + mi * (NB - 1 - j) + (i - j - 1);
}
constexpr int g_tile_count(int NB) { return NB * (NB - 1); }

}  // namespace pf
