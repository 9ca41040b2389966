// State-passing scan fused with the intra-chunk readout: step 3 of Section 3 of ParallelFlow
// (arXiv 2504.00492) as a sequential hand-over of S from chunk to chunk.
//
// Rows of S evolve independently (the recurrence of Section 3.1 multiplies S from the right),
// so a workgroup owns TV rows of S (a tile of d_v) of one (b, h) and walks the chunks; d_v is a
// run-time size (any multiple of the tile), only d = d_k is a template parameter.  Per
// chunk, with T = (Id + G)^{-1} and P = Mbar (.) Q K^T from the chunk-flow kernel:
//     R     = beta (.) (V - K S_c^T)      n x TV       (the chunk's values seen from the incoming state)
//     U_eff = T R                         n x TV       (= U' - W S_c^T: U + W S_0^T of Theorem 3.2, sign folded)
//     O_c   = Q S_c^T + P U_eff           chunk x TV   (discrete flow of Section 3.1 cut at each token)
//     S_c+1 = S_c + U_eff^T K             TV x d       (S_1 of Theorem 3.2)
//
// Only R -> U_eff -> S_c+1 is a chain from one chunk to the next; the readout O_c hangs off it.
// The workgroup therefore has two kinds of wavefronts, one of each per SIMD:
//
//   state waves (0..3)  run the chain: R (interval 0), U_eff (interval 1), S update (interval 2).
//                       Their global loads are their own T tiles, straight into MFMA operand
//                       registers, two chunks ahead (n <= 128; one for n = 256).  For n <= 128 they also compute O: S and
//                       U_eff are already in their registers as operands of the chain, and Q
//                       of a wave's token tiles is loaded straight into operand registers,
//                       so Q S^T and U_eff^T P^T cost no LDS reads.
//   io waves (4..7)     do everything that can be late or early: staging of the next chunk's K,
//                       V tile, beta from registers into LDS and the loads of the chunks after
//                       it (spread over the intervals), the coalesced copy of the previous O tile
//                       to global memory, and for n = 256 (where the state waves have no
//                       registers to spare) Q S^T (interval 0) and U_eff^T P^T (interval 2).
//                       Their load-issue stalls and LDS stores overlap the chain.
//
// S^T lives in fp32 accumulators of the state waves (wave w owns d_k rows [w d/4, (w+1) d/4)); a
// bf16 copy in LDS ([d_v][d_k]) feeds the MFMA operands of the next chunk.  K is read from LDS
// both row-wise (K S^T) and, through the LDS transposing read, column-wise (K^T U_eff); the V
// tile is read transposed into accumulator layout.  R and U_eff go through LDS once each
// ([d_v][n]: accumulator tiles are 4 consecutive tokens of one feature, i.e. 8-byte writes).  O
// is computed transposed (rows = d_v) so that a lane ends up with 4 consecutive features of one
// token.  K is needed in intervals 0 and 2, so the next chunk's K can only be staged during
// interval 1 into a second buffer; where two K buffers do not fit LDS (n = 256 with d = 128) a
// fourth interval is opened at the end of the step in which the io waves overwrite K in place.
// V, Q, beta, the state copy and the O tile are each written in one interval and read in another
// and need one buffer.
//
// The wave id is a compile-time constant of each wave's code (the kernel branches once on it):
// the triangular bounds of T R and of the causal readout then prune whole MFMAs and loads at
// compile time, leaving straight-line code in which LDS reads can be scheduled ahead of the
// MFMAs that use them.  Every fetch is unconditional, the last step re-fetches its own chunk.
#include "pf_internal.h"
#include "pf_common.h"
#include "pf_layout.h"

#include <atomic>

#include <type_traits>

namespace pf {

#define LDS_FENCE() asm volatile("" ::: "memory")

constexpr int kScanRoleWaves = 4;                       // waves per role
constexpr int kScanRoleThreads = 64 * kScanRoleWaves;
constexpr int kScanThreads = 2 * kScanRoleThreads;

// GEN: general drivers (A, Atil, B) of Section 3.1 instead of the delta mapping.  The state is
// multiplied by A rows in interval 0 and updated with B rows in interval 2, so a "K buffer" then
// holds two n x d planes: B first (where K sits otherwise), then A.
template <int D, int N, int C, int TV, bool GEN = false>
struct ScanLds {
    static constexpr int KP = D + 8;   // pitch of a row of K
    static constexpr int VP = TV + 8;  // pitch of a row (virtual token) of the V tile
    static constexpr int SP = D + 8;   // pitch of a row of the bf16 state copy
    static constexpr int UP = N + 8;   // pitch of a row of R^T / U_eff^T
    static constexpr int OP = TV + 8;  // pitch of a row (one token) of the staged O tile
    static constexpr size_t szK = (size_t)(GEN ? 2 : 1) * N * KP * 2;
    static constexpr size_t rest = (size_t)N * VP * 2 + (size_t)N * 4 +
                                   (size_t)TV * SP * 2 + (size_t)2 * TV * UP * 2 + (size_t)C * OP * 2;
    static constexpr bool kDoubleK = 2 * szK + rest <= (size_t)kMaxLdsBytes;
    static constexpr size_t oKs = 0;
    static constexpr size_t oVs = oKs + (kDoubleK ? 2 : 1) * szK;
    static constexpr size_t oBs = oVs + (size_t)N * VP * 2;
    static constexpr size_t oSb = oBs + (size_t)N * 4;
    static constexpr size_t oRs = oSb + (size_t)TV * SP * 2;
    static constexpr size_t oUe = oRs + (size_t)TV * UP * 2;
    static constexpr size_t oOb = oUe + (size_t)TV * UP * 2;
    static constexpr size_t total = oOb + (size_t)C * OP * 2;
};

// RO: the readout O is wanted (false: only the state is advanced, for the per-segment passes of
// the segment-parallel scan).
template <int D, int N, int C, int TV, bool RO, bool GEN = false>
__global__ __launch_bounds__(kScanThreads) void scan_kernel(
    const bf16 *__restrict__ Q, const bf16 *__restrict__ K, const bf16 *__restrict__ V,
    const bf16 *__restrict__ beta, const bf16 *__restrict__ Tt, const bf16 *__restrict__ Pt,
    const float *S0, bf16 *__restrict__ O, float *SL, int nchains, int NC, int tail, int vmul, int s0mul, int dv)
{
    // With GEN, K is the array of B rows, `beta` the array of A rows (n x d each) and V the array
    // of Atil rows: R = Atil + A S^T, U_eff = T R, S += U_eff^T B, O = Q S^T + P U_eff.
    using Ld = ScanLds<D, N, C, TV, GEN>;
    constexpr int KBUF = (int)(Ld::szK / 2);   // elements of one K buffer (both planes with GEN)
    constexpr int R = N / C;
    constexpr int NKS = D / 32;        // k-steps over d
    constexpr int NKT = N / 32;        // k-steps over the chunk's virtual tokens
    constexpr int NNT = TV / 16;       // 16-wide tiles over this workgroup's d_v rows
    constexpr int MT = N / 16;         // 16-row tiles of virtual tokens
    constexpr int CT = C / 16;         // 16-row tiles of tokens
    constexpr int MPW = D / 64;        // d_k tiles (16 rows of S^T) owned by one state wave
    constexpr int M1 = MT / 4;         // 16-row tiles of R / U_eff per state wave
    constexpr int T2 = (CT + 3) / 4;   // 16-token tiles of O per wave of a role (waves beyond CT own none)
    constexpr int KP = Ld::KP, VP = Ld::VP, SP = Ld::SP, UP = Ld::UP, OP = Ld::OP;
    constexpr int NTHR = kScanRoleThreads;
    constexpr bool kDoubleK = Ld::kDoubleK;
    // Who computes O: the state waves when their register budget allows (they already hold S and
    // U_eff as operands, so it costs them no LDS reads but Q), else the io waves.
    // Register sets for the operands that come straight from global memory: two (two blocks of
    // loads in flight) where the registers allow, else one.
    // (measured on blocks of 64 virtual tokens, 64 heads x 4096 / 32 heads x 65536 tokens: one set
    // 0.144 / 1.90 ms, two sets 0.136 / 1.79 ms, four sets 0.142 / 2.07 ms)
    constexpr int kSets = (!GEN && N <= 128 && !(D == 128 && N == 128 && C == 128 && TV == 32)) ? 2 : 1;
    // Recomputing the per-lane offsets every step costs about 100 integer instructions per wave
    // and step but keeps them out of the registers.  Where registers are plentiful (blocks of 64
    // virtual tokens with 32-row tiles, or d = 64) hoisting them wins: 64 heads x 4096 tokens,
    // d = 128: scan 0.130 against 0.136 ms; d = 64: 0.0276 against 0.0292 ms.  With 16-row tiles at
    // d = 128 it loses (1.85 against 1.78 ms on 32 heads x 65536 tokens), with 128 virtual tokens
    // per block too (0.410 against 0.398 ms), and the 32-row instances there would spill.
    constexpr bool kLaunder = !(N <= 64 && (TV == 32 || D == 64));
    constexpr bool kStateReadout = RO && N <= 128;
    constexpr bool kIoReadout = RO && N > 128;
    static_assert(D % 64 == 0 && TV % 16 == 0 && N % 32 == 0, "tile shapes");
    static_assert(MT % 4 == 0 && (CT % 4 == 0 || CT < 4), "tiles are dealt evenly, or at most one token tile per wave");
    static_assert(N <= NTHR, "beta of a chunk is fetched by one pass");

    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16 *Ks = reinterpret_cast<bf16 *>(smem + Ld::oKs);
    bf16 *Vs = reinterpret_cast<bf16 *>(smem + Ld::oVs);
    float *bs = reinterpret_cast<float *>(smem + Ld::oBs);
    bf16 *Sb = reinterpret_cast<bf16 *>(smem + Ld::oSb);
    bf16 *Rs = reinterpret_cast<bf16 *>(smem + Ld::oRs);
    bf16 *Ue = reinterpret_cast<bf16 *>(smem + Ld::oUe);
    bf16 *Ob = reinterpret_cast<bf16 *>(smem + Ld::oOb);

    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane0 = threadIdx.x & 63;

    // Workgroups of one (b, h) are nchains apart in blockIdx, hence on the same XCD (block ids
    // go round-robin over the 8 XCDs) and share that XCD's L2 for K, Q, T and P, which they all read.
    const int tile = blockIdx.x / nchains;
    const size_t chain = blockIdx.x % nchains;
    const int dv0 = tile * TV;
    const size_t c0 = chain * (size_t)NC;
    // A head holds NC whole blocks followed by `tail` tokens that another kernel takes: in Q, K,
    // V, beta, O this head starts chain * tail tokens after its place in the compact numbering.
    // vmul = 0 makes every block of every chain read the same n x d block at V (a block of
    // zeros turns the kernel into the propagator of the transitions alone); s0mul = 0 makes
    // every chain start from the same d x d matrix at S0 (the identity, for that propagator).
    Q += chain * (size_t)tail * D;
    K += chain * (size_t)tail * R * D;
    V += (size_t)vmul * chain * (size_t)tail * R * dv;
    beta += chain * (size_t)tail * R * (GEN ? D : 1);
    if (O) O += chain * (size_t)tail * dv;

    // ------------------------------------------------------------------ state waves
    auto state_wave = [&](auto Wc) {
        constexpr int W = decltype(Wc)::value;
        int lane = lane0, r16 = lane & 15, g = lane >> 4;

        // rows of U_eff owned by this wave: tiles W and 7 - W of every group of 8 (evens out
        // the triangular amount of work of T R); one tile per wave when there are only 4
        constexpr auto row_tile = [](int i) constexpr { return MT >= 8 ? ((i & 1) ? 8 * (i >> 1) + 7 - W : 8 * (i >> 1) + W) : W + 4 * i; };

        f32x4 sacc[MPW][NNT];
#pragma unroll
        for (int a = 0; a < MPW; ++a)
#pragma unroll
            for (int nt = 0; nt < NNT; ++nt) {
                const int mt = W * MPW + a;
                f32x4 v = {0.f, 0.f, 0.f, 0.f};
                if (S0) v = *reinterpret_cast<const f32x4 *>(S0 + (size_t)s0mul * chain * (size_t)dv * D +
                                                             (size_t)(dv0 + 16 * nt + r16) * D + 16 * mt + 4 * g);
                sacc[a][nt] = v;
                st4(&Sb[(16 * nt + r16) * SP + 16 * mt + 4 * g], cvt4(v));
            }

        // readout by the state waves (kStateReadout): token tiles of O owned by this wave, W and
        // (with 8 tiles) 7 - W; token tile tt sees virtual tokens < R (16 tt + 16)
        constexpr auto tok_tile = [](int i) constexpr { return CT >= 8 ? ((i & 1) ? 8 * (i >> 1) + 7 - W : 8 * (i >> 1) + W) : W + 4 * i; };
        // (a chunk of fewer than 64 tokens has fewer tiles than waves: the waves beyond own none)
        constexpr auto ksteps_of = [](int tt) constexpr { return tt < CT ? (R * (16 * tt + 16) + 31) / 32 : 0; };
        // Every operand that comes straight from global memory has two register sets: block ch
        // uses set ch & 1 and, right after its last use, requests block ch + 2 into it, so that
        // two blocks' worth of loads are in flight (one block's worth does not cover the latency
        // of the memory system at the rate a CU can pull data in).
        bf16x8 p2[kSets][T2][NKT]; // P tiles of this wave's token tiles (those the causal mask keeps)
        auto fetch_p = [&](size_t cid, auto Sc) {
            constexpr int S = decltype(Sc)::value % kSets;
            const bf16 *Pc = Pt + cid * (size_t)C * N;
#pragma unroll
            for (int i = 0; i < T2; ++i) {
                const int tt = tok_tile(i);
#pragma unroll
                for (int kt = 0; kt < NKT; ++kt)
                    if (kt < ksteps_of(tt)) p2[S][i][kt] = ld8(Pc + full_tile_offset(NKT, tt, kt) + lane * 8);
            }
        };

        // Q of this wave's token tiles, straight from global memory in B-operand form (16 rows x
        // 64 bytes per load: only a few loads per step, so the poor coalescing does not matter)
        bf16x8 bQ[kSets][T2][NKS];
        auto fetch_q = [&](size_t cid, auto Sc) {
            constexpr int S = decltype(Sc)::value % kSets;
            const bf16 *Qc = Q + cid * (size_t)C * D;
#pragma unroll
            for (int i = 0; i < T2; ++i)
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks)
                    if (tok_tile(i) < CT) bQ[S][i][ks] = ld8(Qc + (size_t)(16 * tok_tile(i) + r16) * D + 32 * ks + 8 * g);
        };

        bf16x8 t1[kSets][M1][NKT]; // T tiles of this wave's rows of U_eff (those below the diagonal)
        auto fetch_t = [&](size_t cid, auto Sc) {
            constexpr int S = decltype(Sc)::value % kSets;
            const bf16 *Tc = Tt + cid * (size_t)N * N;
#pragma unroll
            for (int i = 0; i < M1; ++i) {
                const int mt = row_tile(i);
#pragma unroll
                for (int kt = 0; kt < NKT; ++kt)
                    if (2 * kt <= mt) t1[S][i][kt] = ld8(Tc + full_tile_offset(NKT, mt, kt) + lane * 8);
            }
        };
        constexpr std::integral_constant<int, 0> kSet0{};
        constexpr std::integral_constant<int, 1> kSet1{};
        if (NC > 0) {
            const size_t c1 = NC > 1 ? c0 + 1 : c0;
            fetch_t(c0, kSet0);
            if constexpr (kStateReadout) {
                fetch_p(c0, kSet0);
                fetch_q(c0, kSet0);
            }
            if constexpr (kSets == 2) {
                fetch_t(c1, kSet1);
                if constexpr (kStateReadout) {
                    fetch_p(c1, kSet1);
                    fetch_q(c1, kSet1);
                }
            }
        }
        __syncthreads();

        auto step = [&](int ch, auto Pc) {
            constexpr int PS = decltype(Pc)::value % kSets;   // register set of this block
            // The lane id is laundered once per step so that the per-lane LDS offsets of the
            // unrolled code below are recomputed where they are used instead of being hoisted
            // out of this loop and held in registers for the whole kernel (kLaunder, see below).
            lane = lane0;
            if constexpr (kLaunder) asm volatile("" : "+v"(lane));
            r16 = lane & 15; g = lane >> 4;
            const size_t cid = c0 + ch;
            const size_t nx = ch + kSets < NC ? cid + kSets : c0 + NC - 1;   // the last steps re-fetch the last block
            const bf16 *Kc = Ks + (kDoubleK ? (ch & 1) * KBUF : 0);
            const bf16 *Ka = GEN ? Kc + N * KP : Kc;                 // rows that multiply the state: K, or A

            // Each interval first issues every LDS read it needs and only then starts its MFMAs
            // (LDS_FENCE keeps the reads from sinking down to their first use), so that the
            // read latency is paid once per interval instead of once per MFMA.

            // ---- interval 0: R = beta (.) (V - K S^T), rows (virtual tokens) dealt to the waves
            f32x4 oacc[T2][NNT];
            {
                bf16x8 bS[NNT][NKS], aK[M1][NKS];
                bf16x4 vt[M1][NNT];
                f32x4 bt[M1];
                // reads in the order the MFMAs below consume them, so that the first products can
                // start while the later operands are still on their way
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    aK[0][ks] = ld8(&Ka[(16 * W + r16) * KP + 32 * ks + 8 * g]);
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt) bS[nt][ks] = ld8(&Sb[(16 * nt + r16) * SP + 32 * ks + 8 * g]);
                }
#pragma unroll
                for (int i = 0; i < M1; ++i) {
                    const int mt = W + 4 * i;
                    if constexpr (!GEN) bt[i] = *reinterpret_cast<const f32x4 *>(&bs[16 * mt + 4 * g]);
                    // V tile read transposed: 4 consecutive tokens of feature 16 nt + r16
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt)
                        vt[i][nt] = lds_read_tr4(&Vs[(16 * mt + 4 * g + (r16 >> 2)) * VP + 16 * nt + 4 * (r16 & 3)]);
                    if (i + 1 < M1) {
#pragma unroll
                        for (int ks = 0; ks < NKS; ++ks)
                            aK[i + 1][ks] = ld8(&Ka[(16 * (W + 4 * (i + 1)) + r16) * KP + 32 * ks + 8 * g]);
                    }
                }
                LDS_FENCE();
#pragma unroll
                for (int i = 0; i < M1; ++i) {
                    const int mt = W + 4 * i;
                    f32x4 acc[NNT];
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                        for (int nt = 0; nt < NNT; ++nt) acc[nt] = mfma16(aK[i][ks], bS[nt][ks], acc[nt]);
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt) {
                        f32x4 rr;
                        if constexpr (GEN) rr = __builtin_convertvector(vt[i][nt], f32x4) + acc[nt];
                        else rr = (__builtin_convertvector(vt[i][nt], f32x4) - acc[nt]) * bt[i];
                        st4(&Rs[(16 * nt + r16) * UP + 16 * mt + 4 * g], cvt4(rr));
                    }
                }
                if constexpr (kStateReadout) {
                    // O^T = S Q^T for this wave's token tiles: the rows of S just read as the B
                    // operand of K S^T are, lane for lane, the A operand here
#pragma unroll
                    for (int i = 0; i < T2; ++i) {
                        if (tok_tile(i) >= CT) continue;
#pragma unroll
                        for (int md = 0; md < NNT; ++md) oacc[i][md] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                            for (int md = 0; md < NNT; ++md) oacc[i][md] = mfma16(bS[md][ks], bQ[PS][i][ks], oacc[i][md]);
                    }
                    fetch_q(nx, Pc);
                }
            }
            __syncthreads();

            // ---- interval 1: U_eff = T R, lower block-triangular, rows dealt so that the waves
            // do equal work.  The R tiles (B operands) are shared by this wave's row tiles.
            {
                constexpr int KMAX = row_tile(M1 - 1) / 2 + 1 > row_tile(0) / 2 + 1 ? row_tile(M1 - 1) / 2 + 1
                                                                                      : row_tile(0) / 2 + 1;
                static_assert(KMAX <= NKT, "k-steps of T R");
                bf16x8 bR[KMAX][NNT];
#pragma unroll
                for (int kt = 0; kt < KMAX; ++kt)
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt)
                        bR[kt][nt] = join(ld4(&Rs[(16 * nt + r16) * UP + 32 * kt + 4 * g]),
                                          ld4(&Rs[(16 * nt + r16) * UP + 32 * kt + 16 + 4 * g]));
                LDS_FENCE();
#pragma unroll
                for (int i = 0; i < M1; ++i) {
                    const int mt = row_tile(i);
                    f32x4 acc[NNT];
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kt = 0; kt < KMAX; ++kt) {
                        if (2 * kt <= mt) {
#pragma unroll
                            for (int nt = 0; nt < NNT; ++nt) acc[nt] = mfma16(t1[PS][i][kt], bR[kt][nt], acc[nt]);
                        }
                    }
#pragma unroll
                    // U_eff^T is stored with the tokens of every 32-block in the order two stacked
                    // accumulator tiles have (position 8 g + e holds token 4 g + e for e < 4 and
                    // 16 + 4 g + e - 4 for e >= 4): 16 consecutive bytes of a row are then one lane's
                    // operand both for K^T U_eff (K^T read in the same order) and for U_eff^T P^T
                    for (int nt = 0; nt < NNT; ++nt)
                        st4(&Ue[(16 * nt + r16) * UP + 32 * (mt >> 1) + 8 * g + 4 * (mt & 1)], cvt4(acc[nt]));
                }
            }
            fetch_t(nx, Pc);
            __syncthreads();

            // ---- interval 2: S^T += K^T U_eff, this wave's d_k rows; K^T comes out of the
            // transposing read.  Done in groups of KG k-steps to bound the registers in flight.
            {
                constexpr int KG = NKT < 4 ? NKT : 4;
#pragma unroll
                for (int k0 = 0; k0 < NKT; k0 += KG) {
                    bf16x8 b[KG][NNT], ak[KG][MPW];
#pragma unroll
                    for (int kk = 0; kk < KG; ++kk) {
                        const int kt = k0 + kk;
#pragma unroll
                        for (int nt = 0; nt < NNT; ++nt) b[kk][nt] = ld8(&Ue[(16 * nt + r16) * UP + 32 * kt + 8 * g]);
#pragma unroll
                        for (int a = 0; a < MPW; ++a) {
                            const bf16 *p = &Kc[(32 * kt + 4 * g + (r16 >> 2)) * KP + 16 * (W * MPW + a) + 4 * (r16 & 3)];
                            ak[kk][a] = join(lds_read_tr4(p), lds_read_tr4(p + 16 * KP));
                        }
                    }
                    LDS_FENCE();
#pragma unroll
                    for (int kk = 0; kk < KG; ++kk)
#pragma unroll
                        for (int a = 0; a < MPW; ++a)
#pragma unroll
                            for (int nt = 0; nt < NNT; ++nt) sacc[a][nt] = mfma16(ak[kk][a], b[kk][nt], sacc[a][nt]);
                    if constexpr (kStateReadout) {
                        // O^T += U_eff^T P^T: the same U_eff registers, now as A operand
#pragma unroll
                        for (int kk = 0; kk < KG; ++kk)
#pragma unroll
                            for (int i = 0; i < T2; ++i)
                                if (k0 + kk < ksteps_of(tok_tile(i))) {
#pragma unroll
                                    for (int md = 0; md < NNT; ++md)
                                        oacc[i][md] = mfma16(b[kk][md], p2[PS][i][k0 + kk], oacc[i][md]);
                                }
                    }
                }
            }
#pragma unroll
            for (int a = 0; a < MPW; ++a)
#pragma unroll
                for (int nt = 0; nt < NNT; ++nt)
                    st4(&Sb[(16 * nt + r16) * SP + 16 * (W * MPW + a) + 4 * g], cvt4(sacc[a][nt]));
            if constexpr (kStateReadout) {
#pragma unroll
                for (int i = 0; i < T2; ++i)
#pragma unroll
                    for (int md = 0; md < NNT; ++md)
                        if (tok_tile(i) < CT) st4(&Ob[(16 * tok_tile(i) + r16) * OP + 16 * md + 4 * g], cvt4(oacc[i][md]));
                fetch_p(nx, Pc);
            }
            if (!kDoubleK) __syncthreads();   // interval 3: the io waves overwrite K in place
            __syncthreads();
        };
        for (int ch = 0; ch < NC; ch += 2) {
            step(ch, kSet0);
            if (ch + 1 < NC) step(ch + 1, kSet1);
        }

        if (SL) {
#pragma unroll
            for (int a = 0; a < MPW; ++a)
#pragma unroll
                for (int nt = 0; nt < NNT; ++nt)
                    *reinterpret_cast<f32x4 *>(SL + chain * (size_t)dv * D + (size_t)(dv0 + 16 * nt + r16) * D +
                                               16 * (W * MPW + a) + 4 * g) = sacc[a][nt];
        }
    };

    // ------------------------------------------------------------------ io waves
    auto io_wave = [&](auto Wc) {
        constexpr int W = decltype(Wc)::value;
        const int tb0 = lane0 + 64 * W;                            // thread index among the io waves
        int tb = tb0, lane = lane0, r16 = lane & 15, g = lane >> 4;

        constexpr int VPR = D / 8;                                 // 16-byte vectors per row of K / Q
        constexpr int KV = (N * D / 8 + NTHR - 1) / NTHR;          // vectors of K per thread
        constexpr int PPR = TV / 8;                                // 16-byte pieces per row of the V tile
        constexpr int VV = (N * PPR + NTHR - 1) / NTHR;            // vectors of the V tile per thread
        constexpr int OV = (C * PPR + NTHR - 1) / NTHR;            // vectors of the O tile per thread
        // Two register sets, as in the state waves: block ch + 1 is staged into LDS during step ch
        // out of set (ch + 1) & 1, which is then refilled with block ch + 3, so that two blocks of K,
        // V tile and beta are on their way at any time.
        bf16x8 kreg[kSets][KV], vreg[kSets][VV], areg[kSets][GEN ? KV : 1];
        bf16 breg[kSets];
        bf16x8 p2[kSets][T2][NKT]; // P tiles of this wave's token tiles (those the causal mask keeps)

        // token tiles of O owned by this wave: W and (with 8 tiles) 7 - W
        constexpr auto tok_tile = [](int i) constexpr { return CT >= 8 ? ((i & 1) ? 8 * (i >> 1) + 7 - W : 8 * (i >> 1) + W) : W + 4 * i; };
        // causal readout: token tile tt sees virtual tokens < R (16 tt + 16)
        constexpr auto ksteps_of = [](int tt) constexpr { return tt < CT ? (R * (16 * tt + 16) + 31) / 32 : 0; };

        // K moves in two halves (vectors [0, KH) and [KH, KV) of every thread) so that its
        // staging and load issue can be spread over two intervals
        constexpr int KH = KV / 2;
        auto fetch_k = [&](size_t cid, int q0, int q1, auto Sc) {
            constexpr int S = decltype(Sc)::value % kSets;
            const bf16 *Kg = K + cid * (size_t)N * D;
#pragma unroll
            for (int q = 0; q < KV; ++q) {
                const int v = tb + NTHR * q;
                if (q >= q0 && q < q1 && ((q + 1) * NTHR <= N * D / 8 || v < N * D / 8)) {
                    kreg[S][q] = ld8(Kg + (size_t)v * 8);
                    if constexpr (GEN) areg[S][q] = ld8(beta + cid * (size_t)N * D + (size_t)v * 8);
                }
            }
        };
        auto fetch_vqb = [&](size_t cid, auto Sc) {
            constexpr int S = decltype(Sc)::value % kSets;
            const bf16 *Vg = V + (size_t)vmul * cid * (size_t)N * dv + dv0;
#pragma unroll
            for (int q = 0; q < VV; ++q) {
                int v = tb + NTHR * q;
                v = v < N * PPR ? v : N * PPR - 1;                 // clamp instead of branching
                vreg[S][q] = ld8(Vg + (size_t)(v / PPR) * dv + (v % PPR) * 8);
            }
            if constexpr (!GEN) breg[S] = beta[cid * (size_t)N + (tb % N)];
        };
        auto fetch_p = [&](size_t cid, auto Sc) {
            constexpr int S = decltype(Sc)::value % kSets;
            const bf16 *Pc = Pt + cid * (size_t)C * N;
#pragma unroll
            for (int i = 0; i < T2; ++i) {
                const int tt = tok_tile(i);
#pragma unroll
                for (int kt = 0; kt < NKT; ++kt)
                    if (kt < ksteps_of(tt)) p2[S][i][kt] = ld8(Pc + full_tile_offset(NKT, tt, kt) + lane * 8);
            }
        };
        // Q of this wave's token tiles, straight from global memory in B-operand form
        bf16x8 bQ[kSets][T2][NKS];
        auto fetch_q = [&](size_t cid, auto Sc) {
            constexpr int S = decltype(Sc)::value % kSets;
            const bf16 *Qc = Q + cid * (size_t)C * D;
#pragma unroll
            for (int i = 0; i < T2; ++i)
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks)
                    if (tok_tile(i) < CT) bQ[S][i][ks] = ld8(Qc + (size_t)(16 * tok_tile(i) + r16) * D + 32 * ks + 8 * g);
        };
        auto stage_k = [&](bf16 *Kd, int q0, int q1, auto Sc) {
            constexpr int S = decltype(Sc)::value % kSets;
#pragma unroll
            for (int q = 0; q < KV; ++q) {
                const int v = tb + NTHR * q;
                if (q >= q0 && q < q1 && ((q + 1) * NTHR <= N * D / 8 || v < N * D / 8)) {
                    st8(&Kd[(v / VPR) * KP + (v % VPR) * 8], kreg[S][q]);
                    if constexpr (GEN) st8(&Kd[N * KP + (v / VPR) * KP + (v % VPR) * 8], areg[S][q]);
                }
            }
        };
        auto stage_vqb = [&](auto Sc) {
            constexpr int S = decltype(Sc)::value % kSets;
#pragma unroll
            for (int q = 0; q < VV; ++q) {
                const int v = tb + NTHR * q;
                if (v < N * PPR) st8(&Vs[(v / PPR) * VP + (v % PPR) * 8], vreg[S][q]);
            }
            if constexpr (!GEN) {
                if (tb < N) bs[tb] = (float)breg[S];
            }
        };
        // the O tile of one chunk (chunk tokens x TV features), LDS -> its rows of O
        auto copy_out = [&](size_t cid) {
            if constexpr (!RO) return;
            bf16 *Oc = O + cid * (size_t)C * dv;
#pragma unroll
            for (int q = 0; q < OV; ++q) {
                const int v = tb + NTHR * q;
                if ((q + 1) * NTHR <= C * PPR || v < C * PPR)
                    st8(Oc + (size_t)(v / PPR) * dv + dv0 + 8 * (v % PPR), ld8(&Ob[(v / PPR) * OP + 8 * (v % PPR)]));
            }
        };

        constexpr std::integral_constant<int, 0> kSet0{};
        constexpr std::integral_constant<int, 1> kSet1{};
        if (NC > 0) {
            const size_t last = c0 + NC - 1;
            const size_t c1 = NC > 1 ? c0 + 1 : last, c2 = NC > 2 ? c0 + 2 : last;
            fetch_k(c0, 0, KV, kSet0);
            fetch_vqb(c0, kSet0);
            if constexpr (kIoReadout) {
                fetch_p(c0, kSet0);
                fetch_q(c0, kSet0);
                if constexpr (kSets == 2) {
                    fetch_p(c1, kSet1);
                    fetch_q(c1, kSet1);
                }
            }
            if constexpr (kSets == 2) {
                fetch_k(c1, 0, KV, kSet1);
                fetch_vqb(c1, kSet1);
            }
            stage_k(Ks, 0, KV, kSet0);
            stage_vqb(kSet0);
            // with one set: block 1 now; with two: block 2 (block 1 is already on its way)
            fetch_k(kSets == 2 ? c2 : c1, 0, KV, kSet0);
            fetch_vqb(kSets == 2 ? c2 : c1, kSet0);
        }
        __syncthreads();

        auto step = [&](int ch, auto Pc) {
            constexpr int PS = decltype(Pc)::value % kSets;                          // set of block ch
            constexpr std::integral_constant<int, (decltype(Pc)::value + 1) % kSets> Nc{};   // set that holds block ch + 1
            tb = tb0;
            if constexpr (kLaunder) asm volatile("" : "+v"(tb));
            lane = tb & 63; r16 = lane & 15; g = lane >> 4;
            const size_t cid = c0 + ch;
            const size_t n2 = ch + kSets < NC ? cid + kSets : c0 + NC - 1;          // block to request into this block's set
            const size_t n3 = ch + 1 + kSets < NC ? cid + 1 + kSets : c0 + NC - 1;  // ... into the next block's set

            // ---- interval 0: previous O tile out; O^T = S Q^T for this wave's token tiles; first
            // half of the next chunk's K into the buffer this step does not read
            if (ch > 0) copy_out(cid - 1);
            f32x4 oacc[T2][NNT];
            if constexpr (kIoReadout) {
                bf16x8 aS[NNT][NKS];
#pragma unroll
                for (int md = 0; md < NNT; ++md)
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks) aS[md][ks] = ld8(&Sb[(16 * md + r16) * SP + 32 * ks + 8 * g]);
                LDS_FENCE();
#pragma unroll
                for (int i = 0; i < T2; ++i) {
                    if (tok_tile(i) >= CT) continue;
#pragma unroll
                    for (int md = 0; md < NNT; ++md) oacc[i][md] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                        for (int md = 0; md < NNT; ++md) oacc[i][md] = mfma16(aS[md][ks], bQ[PS][i][ks], oacc[i][md]);
                }
                fetch_q(n2, Pc);
            }
            bf16 *Knext = Ks + (kDoubleK ? ((ch + 1) & 1) * KBUF : 0);
            if (kDoubleK) {
                stage_k(Knext, 0, KH, Nc);
                fetch_k(n3, 0, KH, Nc);
            }
            __syncthreads();

            // ---- interval 1: next chunk's V tile and beta registers -> LDS, the chunk after the
            // one after it on its way
            stage_vqb(Nc);
            fetch_vqb(n3, Nc);
            __syncthreads();

            // ---- interval 2: O^T += U_eff^T P^T, O tile to LDS
            if constexpr (kIoReadout) {
                constexpr int KMAX = ksteps_of(tok_tile(T2 - 1)) > ksteps_of(tok_tile(0)) ? ksteps_of(tok_tile(T2 - 1))
                                                                                          : ksteps_of(tok_tile(0));
                constexpr int KM = KMAX < 1 ? 1 : (KMAX < NKT ? KMAX : NKT);
                bf16x8 aU[KM][NNT];
#pragma unroll
                for (int kt = 0; kt < KM; ++kt)
#pragma unroll
                    for (int md = 0; md < NNT; ++md)
                        aU[kt][md] = ld8(&Ue[(16 * md + r16) * UP + 32 * kt + 8 * g]);
                LDS_FENCE();
#pragma unroll
                for (int i = 0; i < T2; ++i) {
                    const int tt = tok_tile(i);
                    if (tt >= CT) continue;
#pragma unroll
                    for (int kt = 0; kt < KM; ++kt)
                        if (kt < ksteps_of(tt)) {
#pragma unroll
                            for (int md = 0; md < NNT; ++md) oacc[i][md] = mfma16(aU[kt][md], p2[PS][i][kt], oacc[i][md]);
                        }
#pragma unroll
                    for (int md = 0; md < NNT; ++md)
                        st4(&Ob[(16 * tt + r16) * OP + 16 * md + 4 * g], cvt4(oacc[i][md]));
                }
            }
            if constexpr (kIoReadout) fetch_p(n2, Pc);
            if (kDoubleK) {
                stage_k(Knext, KH, KV, Nc);
                fetch_k(n3, KH, KV, Nc);
            } else {
                // ---- interval 3: K of the next chunk replaces this chunk's in place
                __syncthreads();
                stage_k(Ks, 0, KV, Nc);
                fetch_k(n3, 0, KV, Nc);
            }
            __syncthreads();
        };
        for (int ch = 0; ch < NC; ch += 2) {
            step(ch, kSet0);
            if (ch + 1 < NC) step(ch + 1, kSet1);
        }
        if (NC > 0) copy_out(c0 + NC - 1);
    };

    switch (wave) {
    case 0: state_wave(std::integral_constant<int, 0>{}); break;
    case 1: state_wave(std::integral_constant<int, 1>{}); break;
    case 2: state_wave(std::integral_constant<int, 2>{}); break;
    case 3: state_wave(std::integral_constant<int, 3>{}); break;
    case 4: io_wave(std::integral_constant<int, 0>{}); break;
    case 5: io_wave(std::integral_constant<int, 1>{}); break;
    case 6: io_wave(std::integral_constant<int, 2>{}); break;
    default: io_wave(std::integral_constant<int, 3>{}); break;
    }
}

// ---------------------------------------------------------------------------- host side
#ifndef PF_SCAN_INSTANCES
#define PF_SCAN_INSTANCES(X) \
    X(64, 64, 64) X(64, 64, 32) X(64, 128, 32) X(64, 128, 64) X(64, 128, 128) X(64, 256, 64) X(64, 256, 128) \
    X(128, 64, 64) X(128, 64, 32) X(128, 128, 32) X(128, 128, 64) X(128, 128, 128) X(128, 256, 64) X(128, 256, 128)
#endif

template <int D, int N, int C, int TV, bool RO, bool GEN = false>
static hipError_t launch_scan_ro(const void *Q, const void *K, const void *V, const void *beta,
                                       const void *Tt, const void *Pt, const float *S0, void *O, float *SL,
                                       int heads, int NC, int tail, int vmul, int s0mul, int dv, hipStream_t stream)
{
    auto kern = scan_kernel<D, N, C, TV, RO, GEN>;
    constexpr size_t lds = ScanLds<D, N, C, TV, GEN>::total;
    static_assert(lds <= kMaxLdsBytes, "scan kernel LDS plan exceeds the CU");
    static std::atomic<uint64_t> armed{0};
    hipError_t e = arm_dynamic_lds(armed, reinterpret_cast<const void *>(kern), lds);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)heads * (dv / TV);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kScanThreads), lds, stream, (const bf16 *)Q,
                       (const bf16 *)K, (const bf16 *)V, (const bf16 *)beta, (const bf16 *)Tt,
                       (const bf16 *)Pt, S0, (bf16 *)O, SL, heads, NC, tail, vmul, s0mul, dv);
    return hipGetLastError();
}

int scan_dv_tile(int heads, int dv, int n)
{
    // 32 rows when that already gives at least one workgroup per CU, else 16 rows (twice the
    // workgroups, half the MFMA work per operand byte).  With n = 256 only the 16-row tile
    // fits LDS next to the chunk's K.
    return (n < 256 && dv % 32 == 0 && (long long)heads * (dv / 32) >= (long long)device_cu_count()) ? 32 : 16;
}

template <int D, int N, int C, int TV>
static hipError_t launch_scan_instance(const void *Q, const void *K, const void *V, const void *beta,
                                       const void *Tt, const void *Pt, const float *S0, void *O, float *SL,
                                       int heads, int NC, int tail, int vmul, int s0mul, int dv, hipStream_t stream)
{
    return O ? launch_scan_ro<D, N, C, TV, true>(Q, K, V, beta, Tt, Pt, S0, O, SL, heads, NC, tail, vmul, s0mul, dv, stream)
             : launch_scan_ro<D, N, C, TV, false>(Q, K, V, beta, Tt, Pt, S0, O, SL, heads, NC, tail, vmul, s0mul, dv, stream);
}

hipError_t launch_chunk_scan(const void *Q, const void *K, const void *V, const void *beta, const void *Tt,
                             const void *Pt, const float *S0, void *O, float *SL, int heads, int L, int d,
                             int r, int chunk, hipStream_t stream, int vmul, int s0mul, int dv)
{
    const int NC = L / chunk, tail = L % chunk;   // the tail tokens of every head are skipped
    const int n = chunk * r;
    if (dv <= 0) dv = d;
    if (dv % 16 != 0 || (long long)heads * (dv / 16) > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool wide = scan_dv_tile(heads, dv, n) == 32;
#define X(DD, NN, CC)                                                                                      \
    if (d == DD && n == NN && chunk == CC) {                                                                \
        if constexpr (NN < 256) {                                                                           \
            if (wide)                                                                                       \
                return launch_scan_instance<DD, NN, CC, 32>(Q, K, V, beta, Tt, Pt, S0, O, SL, heads, NC, tail, vmul, s0mul, dv, stream); \
        }                                                                                                   \
        return launch_scan_instance<DD, NN, CC, 16>(Q, K, V, beta, Tt, Pt, S0, O, SL, heads, NC, tail, vmul, s0mul, dv, stream);   \
    }
    PF_SCAN_INSTANCES(X)
#undef X
    return hipErrorInvalidValue;
}

hipError_t launch_chunk_scan_general(const void *Q, const void *A, const void *Atil, const void *Bm, const void *Tt,
                                     const void *Pt, const float *S0, void *O, float *SL, int heads, int L, int d,
                                     int dv, int r, int chunk, hipStream_t stream)
{
    const int NC = L / chunk, tail = L % chunk;   // the tail tokens of every head are skipped
    const int n = chunk * r;
    if (!O || dv <= 0 || dv % 16 != 0 || (long long)heads * (dv / 16) > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool wide = scan_dv_tile(heads, dv, n) == 32;
    // operand slots of the kernel: K <- B rows, beta <- A rows, V <- Atil rows
#define X(DD, NN, CC)                                                                                      \
    if constexpr (NN <= 128) {                                                                              \
        if (d == DD && n == NN && chunk == CC) {                                                            \
            if (wide)                                                                                       \
                return launch_scan_ro<DD, NN, CC, 32, true, true>(Q, Bm, Atil, A, Tt, Pt, S0, O, SL, heads, NC, tail, 1, 1, dv, stream); \
            return launch_scan_ro<DD, NN, CC, 16, true, true>(Q, Bm, Atil, A, Tt, Pt, S0, O, SL, heads, NC, tail, 1, 1, dv, stream);     \
        }                                                                                                   \
    }
    PF_SCAN_INSTANCES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace pf
