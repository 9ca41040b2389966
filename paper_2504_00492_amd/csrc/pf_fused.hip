// Fused forward: steps 2 and 3 of Section 3 of ParallelFlow (arXiv 2504.00492) in one kernel.
// The flow of a block (Theorem 3.2) is built inside the workgroup that scans the block, so the
// compact form T and the masked readout matrix P never leave the compute unit: HBM sees q, k, v,
// beta once and o once, as long as the d_v tiles of a head stay in step (see below).
//
// Rows of S evolve independently (the recurrence of Section 3.1 multiplies S from the right), so a
// workgroup owns TV rows of S (a tile of d_v) of one (b, h) and walks the blocks.  The d_v tiles of
// a head run side by side on one XCD and share the head's K, Q, beta through its L2; each of
// them builds T and P for itself (the price of keeping them on chip).
//
// Per block of n = block * r virtual tokens, in delta variables (Remark in Section 3.1), with M strict
// and Mbar inclusive in time:
//     G     = M (.) diag(beta) K K^T,   T = (Id + G)^{-1}           (Id - M (.) A B^T of Theorem 3.2, inverted)
//     P     = Mbar (.) Q K^T
//     R     = beta (.) (V - K S_c^T)      n x TV
//     U_eff = T R                         n x TV       (= U + W S_0^T of Theorem 3.2, sign folded)
//     O_c   = Q S_c^T + P U_eff           block x TV   (discrete flow of Section 3.1 cut at each token)
//     S_c+1 = S_c + U_eff^T K             TV x d       (S_1 of Theorem 3.2)
//
// Three kinds of wavefronts, one of each per SIMD (twelve waves, 168 registers each), meet at
// three barriers per block:
//
//   state waves (0..3)  run the chain R (interval 0), U_eff (interval 1), S update (interval 2) and
//                       the readout that hangs off it; S^T lives in their fp32 accumulators for the
//                       whole sequence.  T and P come from LDS, Q straight from global memory in
//                       operand form, one block ahead.
//   gram waves (4..7)   work one block ahead of the chain.  Interval 0: P of the block the chain
//                       is on goes from their registers to LDS.  Interval 1: Gram of the next
//                       block (K K^T below the diagonal as operand tiles of -G^T in LDS, P = Q K^T
//                       into registers).  Interval 2: their share of the block substitution.
//   aux waves (8..11)   stage K, V, beta of the next block through registers into LDS and copy
//                       the previous O tile out (interval 0), invert the diagonal 32-blocks of
//                       Id + G (interval 1), and take the other share of the substitution
//                       (interval 2).
//
// The substitution is Proposition 3.3 on the transposed system: column blocks of T are slices
// kept in registers as B operands, finished tiles go to LDS in the A-operand form the chain reads.
//
// Measured on MI355X (d = 128, r = 2): 64 heads of 4096 tokens, 32-row tiles: 1.01 times the
// minimal HBM bytes, 0.22 ms, the same time as the two-kernel path; 32 heads of 65536 tokens,
// 16-row tiles: 1.4 to 1.8 times the minimal bytes (the eight tiles of a head drift apart over
// 1024 blocks and miss each other's K and Q in L2), 2.8 ms against 2.3 ms.  A compute unit does the
// flow of its block D / TV times over, and the chain, the Gram and the substitution all draw on
// the same LDS ports (MFMA pipe busy 31 %, LDS 56 % of the cycles).  It serves callers that
// have no workspace.
//
// T_jj (32 x 32): the two 16 x 16 diagonal inverses are (Id + M)(Id + M^2)(Id + M^4)(Id + M^8) with
// M = -N strictly lower (nilpotent of index <= 16), evaluated on MFMAs (contraction length 16) without leaving
// registers: an accumulator tile of X is the B operand of X and the A operand of X^T, so X and X^T
// are carried together.  T_21 = T_22 M_21 T_11 the same way.
#include "pf_internal.h"
#include "pf_common.h"
#include "pf_layout.h"

#include <atomic>
#include <type_traits>

namespace pf {

#define LDS_FENCE() asm volatile("" ::: "memory")

constexpr int kFusedRoleWaves = 4;                       // waves per role
constexpr int kFusedRoleThreads = 64 * kFusedRoleWaves;
constexpr int kFusedThreads = 3 * kFusedRoleThreads;     // state, gram and aux waves

// 16 x 16 x 16 product.  The instruction takes its bf16 operands as 16-bit integers; the pair of
// packed conversions is made opaque before that reinterpretation, otherwise the conversion is done
// element by element and repacked.
__device__ __forceinline__ f32x4 mfma16k(bf16x4 a, bf16x4 b, f32x4 c)
{
    u32x2 ua = __builtin_bit_cast(u32x2, a), ub = __builtin_bit_cast(u32x2, b);
    asm volatile("" : "+v"(ua), "+v"(ub));
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, ua), __builtin_bit_cast(s16x4, ub), c, 0, 0, 0);
}

template <int D, int N, int C, int TV>
struct FusedLds {
    static constexpr int R = N / C, NB = N / 32, MT = N / 16, CT = C / 16;
    static constexpr int KP = D + 8;   // pitch of a row of K
    static constexpr int VP = TV + 8;  // pitch of a row (virtual token) of the V tile
    static constexpr int SP = D + 8;   // pitch of a row of the bf16 state copy
    static constexpr int UP = N + 8;   // pitch of a row of R^T / U_eff^T
    static constexpr int OP = TV + 8;  // pitch of a row (one token) of the staged O tile
    static constexpr size_t szK = (size_t)N * KP * 2;
    static constexpr size_t oKs = 0;                                   // K, two slots
    static constexpr size_t oBs = oKs + 2 * szK;                       // beta (fp32), two slots
    static constexpr size_t oVs = oBs + 2 * (size_t)N * 4;             // V tile
    static constexpr size_t oSb = oVs + (size_t)N * VP * 2;            // bf16 copy of the state tile
    static constexpr size_t oRs = oSb + (size_t)TV * SP * 2;           // R^T
    static constexpr size_t oUe = oRs + (size_t)TV * UP * 2;           // U_eff^T
    static constexpr size_t oOb = oUe + (size_t)TV * UP * 2;           // O tile
    static constexpr size_t oTl = oOb + (size_t)C * OP * 2;            // T tiles (compact)
    static constexpr size_t oPl = oTl + (size_t)t_tile_count(MT) * 1024;       // P tiles (compact)
    static constexpr size_t oGs = oPl + (size_t)p_tile_count(R, CT) * 1024;    // -G^T tiles
    static constexpr size_t oTs = oGs + (size_t)g_tile_count(NB) * 1024;       // T_jj^T tiles
    static constexpr size_t total = oTs + (size_t)2 * NB * 1024;
};

template <int D, int N, int C, int TV>
__global__ __launch_bounds__(kFusedThreads) void fused_kernel(
    const bf16 *__restrict__ Q, const bf16 *__restrict__ K, const bf16 *__restrict__ V,
    const bf16 *__restrict__ beta, const float *S0, bf16 *__restrict__ O, float *SL,
    bf16 *__restrict__ Tdump, bf16 *__restrict__ Pdump, int nchains, int NC, int tail, int mask_shift)
{
    using Ld = FusedLds<D, N, C, TV>;
    constexpr int R = N / C;
    constexpr int NKS = D / 32;        // k-steps over d
    constexpr int NKT = N / 32;        // k-steps over the block's virtual tokens
    constexpr int NNT = TV / 16;       // 16-wide tiles over this workgroup's d_v rows
    constexpr int MT = N / 16;         // 16-row tiles of virtual tokens
    constexpr int CT = C / 16;         // 16-row tiles of tokens
    constexpr int NB = N / 32;         // 32-row blocks of the substitution
    constexpr int MPW = D / 64;        // d_k tiles (16 rows of S^T) owned by one state wave
    constexpr int M1 = MT / 4;         // 16-row tiles of R / U_eff per state wave
    constexpr int T2 = (CT + 3) / 4;   // 16-token tiles of O per state wave (waves beyond CT own none)
    constexpr int KP = Ld::KP, VP = Ld::VP, SP = Ld::SP, UP = Ld::UP, OP = Ld::OP;
    constexpr int NTHR = kFusedRoleThreads;
    static_assert(D % 64 == 0 && TV % 16 == 0 && N % 32 == 0 && C % 16 == 0 && 32 % R == 0, "tile shapes");
    static_assert(N == 64 || N == 128, "flow blocks of 64 or 128 virtual tokens");
    static_assert(MT % 4 == 0 && (CT % 4 == 0 || CT < 4), "tiles are dealt evenly, or at most one token tile per wave");
    static_assert((N * D / 8) % NTHR == 0, "K of a block is staged in whole passes");

    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16 *Ks = reinterpret_cast<bf16 *>(smem + Ld::oKs);
    float *bs = reinterpret_cast<float *>(smem + Ld::oBs);
    bf16 *Vs = reinterpret_cast<bf16 *>(smem + Ld::oVs);
    bf16 *Sb = reinterpret_cast<bf16 *>(smem + Ld::oSb);
    bf16 *Rs = reinterpret_cast<bf16 *>(smem + Ld::oRs);
    bf16 *Ue = reinterpret_cast<bf16 *>(smem + Ld::oUe);
    bf16 *Ob = reinterpret_cast<bf16 *>(smem + Ld::oOb);
    bf16 *Tl = reinterpret_cast<bf16 *>(smem + Ld::oTl);
    bf16 *Pl = reinterpret_cast<bf16 *>(smem + Ld::oPl);
    bf16 *Gs = reinterpret_cast<bf16 *>(smem + Ld::oGs);
    bf16 *Ts = reinterpret_cast<bf16 *>(smem + Ld::oTs);

    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane0 = threadIdx.x & 63;

    // The d_v tiles of one (b, h) take consecutive places on one XCD (block ids go round-robin over
    // the 8 XCDs): they start together and share K, Q and beta through that XCD's L2.
    constexpr int NTL = D / TV;
    int tile, chain_i;
    if ((nchains & 7) == 0) {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        tile = slot % NTL;
        chain_i = (slot / NTL) * 8 + xcd;
    } else {
        tile = blockIdx.x / nchains;
        chain_i = blockIdx.x % nchains;
    }
    const size_t chain = (size_t)chain_i;
    const int dv0 = tile * TV;
    const size_t c0 = chain * (size_t)NC;
    // A head holds NC whole blocks followed by `tail` tokens that another kernel takes: in Q, K,
    // V, beta, O this head starts chain * tail tokens after its place in the compact numbering.
    Q += chain * (size_t)tail * D;
    K += chain * (size_t)tail * R * D;
    V += chain * (size_t)tail * R * D;
    beta += chain * (size_t)tail * R;
    O += chain * (size_t)tail * D;

    // ------------------------------------------------------------------ state waves
    auto state_wave = [&](auto Wc) {
        constexpr int W = decltype(Wc)::value;
        int lane = lane0, r16 = lane & 15, g = lane >> 4;

        // rows of U_eff owned by this wave: tiles W and 7 - W of every group of 8 (evens out
        // the triangular amount of work of T R); one tile per wave when there are only 4
        constexpr auto row_tile = [](int i) constexpr { return MT >= 8 ? ((i & 1) ? 8 * (i >> 1) + 7 - W : 8 * (i >> 1) + W) : W + 4 * i; };
        // token tiles of O owned by this wave, W and (with 8 tiles) 7 - W
        constexpr auto tok_tile = [](int i) constexpr { return CT >= 8 ? ((i & 1) ? 8 * (i >> 1) + 7 - W : 8 * (i >> 1) + W) : W + 4 * i; };
        constexpr auto ksteps_of = [](int tt) constexpr { return tt < CT ? p_ksteps(R, tt) : 0; };

        f32x4 sacc[MPW][NNT];
#pragma unroll
        for (int a = 0; a < MPW; ++a)
#pragma unroll
            for (int nt = 0; nt < NNT; ++nt) {
                const int mt = W * MPW + a;
                f32x4 v = {0.f, 0.f, 0.f, 0.f};
                if (S0) v = *reinterpret_cast<const f32x4 *>(S0 + chain * (size_t)D * D +
                                                             (size_t)(dv0 + 16 * nt + r16) * D + 16 * mt + 4 * g);
                sacc[a][nt] = v;
                st4(&Sb[(16 * nt + r16) * SP + 16 * mt + 4 * g], cvt4(v));
            }

        // Q of this wave's token tiles, straight from global memory in B-operand form; right after
        // its use in interval 0 the next block's is requested
        bf16x8 bQ[T2][NKS];
        auto fetch_q = [&](size_t cid) {
            const bf16 *Qc = Q + cid * (size_t)C * D;
#pragma unroll
            for (int i = 0; i < T2; ++i)
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks)
                    if (tok_tile(i) < CT) bQ[i][ks] = ld8(Qc + (size_t)(16 * tok_tile(i) + r16) * D + 32 * ks + 8 * g);
        };
        fetch_q(c0);
        // the flow waves' first round (block 0: K to LDS, Gram, T)
        __syncthreads();
        __syncthreads();
        __syncthreads();

        auto step = [&](int ch) {
            // The lane id is laundered once per step so that the per-lane LDS offsets of the
            // unrolled code below are recomputed where they are used instead of being hoisted
            // out of this loop and held in registers for the whole kernel.
            lane = lane0;
            // With 32 rows of S per workgroup the registers are short: the lane id is made opaque once
            // per step, so that the per-lane LDS offsets are recomputed where they are used instead of
            // being held for the whole kernel (the 16-row instance keeps them: fewer instructions).
            if constexpr (NNT >= 2) asm volatile("" : "+v"(lane));
            r16 = lane & 15; g = lane >> 4;
            const size_t cid = c0 + ch;
            const size_t nx = ch + 1 < NC ? cid + 1 : cid;   // the last step re-fetches its own block
            const bf16 *Kc = Ks + (ch & 1) * N * KP;      // block ch sits in LDS slot ch & 1
            const float *bc = bs + (ch & 1) * N;

            // ---- interval 0: R = beta (.) (V - K S^T), rows (virtual tokens) dealt to the waves
            f32x4 oacc[T2][NNT];
            {
                bf16x8 bS[NNT][NKS], aK[M1][NKS];
                bf16x4 vt[M1][NNT];
                f32x4 bt[M1];
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    aK[0][ks] = ld8(&Kc[(16 * W + r16) * KP + 32 * ks + 8 * g]);
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt) bS[nt][ks] = ld8(&Sb[(16 * nt + r16) * SP + 32 * ks + 8 * g]);
                }
#pragma unroll
                for (int i = 0; i < M1; ++i) {
                    const int mt = W + 4 * i;
                    bt[i] = *reinterpret_cast<const f32x4 *>(&bc[16 * mt + 4 * g]);
                    // V tile read transposed: 4 consecutive tokens of feature 16 nt + r16
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt)
                        vt[i][nt] = lds_read_tr4(&Vs[(16 * mt + 4 * g + (r16 >> 2)) * VP + 16 * nt + 4 * (r16 & 3)]);
                    if (i + 1 < M1) {
#pragma unroll
                        for (int ks = 0; ks < NKS; ++ks)
                            aK[i + 1][ks] = ld8(&Kc[(16 * (W + 4 * (i + 1)) + r16) * KP + 32 * ks + 8 * g]);
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
                        f32x4 rr = (__builtin_convertvector(vt[i][nt], f32x4) - acc[nt]) * bt[i];
                        st4(&Rs[(16 * nt + r16) * UP + 16 * mt + 4 * g], cvt4(rr));
                    }
                }
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
                        for (int md = 0; md < NNT; ++md) oacc[i][md] = mfma16(bS[md][ks], bQ[i][ks], oacc[i][md]);
                }
                fetch_q(nx);
            }
            __syncthreads();

            // ---- interval 1: U_eff = T R, lower block-triangular, rows dealt so that the waves
            // do equal work.  The R tiles (B operands) are shared by this wave's row tiles.
            {
                constexpr int KMAX = row_tile(M1 - 1) / 2 + 1 > row_tile(0) / 2 + 1 ? row_tile(M1 - 1) / 2 + 1
                                                                                      : row_tile(0) / 2 + 1;
                static_assert(KMAX <= NKT, "k-steps of T R");
                bf16x8 bR[KMAX][NNT], t1[M1][KMAX];
#pragma unroll
                for (int kt = 0; kt < KMAX; ++kt) {
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt)
                        bR[kt][nt] = join(ld4(&Rs[(16 * nt + r16) * UP + 32 * kt + 4 * g]),
                                          ld4(&Rs[(16 * nt + r16) * UP + 32 * kt + 16 + 4 * g]));
#pragma unroll
                    for (int i = 0; i < M1; ++i)
                        if (2 * kt <= row_tile(i)) t1[i][kt] = ld8(&Tl[((size_t)t_tile_index(row_tile(i), kt) * 64 + lane) * 8]);
                }
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
                            for (int nt = 0; nt < NNT; ++nt) acc[nt] = mfma16(t1[i][kt], bR[kt][nt], acc[nt]);
                        }
                    }
                    // U_eff^T is stored with the tokens of every 32-block in the order two stacked
                    // accumulator tiles have (position 8 g + e holds token 4 g + e for e < 4 and
                    // 16 + 4 g + e - 4 for e >= 4): 16 consecutive bytes of a row are then one lane's
                    // operand both for K^T U_eff (K^T read in the same order) and for U_eff^T P^T
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt)
                        st4(&Ue[(16 * nt + r16) * UP + 32 * (mt >> 1) + 8 * g + 4 * (mt & 1)], cvt4(acc[nt]));
                }
            }
            __syncthreads();

            // ---- interval 2: S^T += K^T U_eff, this wave's d_k rows; K^T comes out of the
            // transposing read.  O^T += U_eff^T P^T reuses the U_eff registers as A operand.
            {
                bf16x8 p2[T2][NKT];
#pragma unroll
                for (int i = 0; i < T2; ++i)
#pragma unroll
                    for (int kt = 0; kt < NKT; ++kt)
                        if (kt < ksteps_of(tok_tile(i)))
                            p2[i][kt] = ld8(&Pl[((size_t)p_tile_index(R, tok_tile(i), kt) * 64 + lane) * 8]);
                constexpr int KG = NNT >= 2 ? 2 : (NKT < 4 ? NKT : 4);   // k-steps per group: bounds the operands in flight
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
#pragma unroll
                    for (int kk = 0; kk < KG; ++kk)
#pragma unroll
                        for (int i = 0; i < T2; ++i)
                            if (k0 + kk < ksteps_of(tok_tile(i))) {
#pragma unroll
                                for (int md = 0; md < NNT; ++md)
                                    oacc[i][md] = mfma16(b[kk][md], p2[i][k0 + kk], oacc[i][md]);
                            }
                }
            }
#pragma unroll
            for (int a = 0; a < MPW; ++a)
#pragma unroll
                for (int nt = 0; nt < NNT; ++nt)
                    st4(&Sb[(16 * nt + r16) * SP + 16 * (W * MPW + a) + 4 * g], cvt4(sacc[a][nt]));
#pragma unroll
            for (int i = 0; i < T2; ++i)
#pragma unroll
                for (int md = 0; md < NNT; ++md)
                    if (tok_tile(i) < CT) st4(&Ob[(16 * tok_tile(i) + r16) * OP + 16 * md + 4 * g], cvt4(oacc[i][md]));
            __syncthreads();
        };
        // (one copy of the step's code: the twelve wavefronts of a workgroup run twelve different
        // instruction streams, and together they have to stay within the instruction cache)
        for (int ch = 0; ch < NC; ++ch) step(ch);

        if (SL) {
#pragma unroll
            for (int a = 0; a < MPW; ++a)
#pragma unroll
                for (int nt = 0; nt < NNT; ++nt)
                    *reinterpret_cast<f32x4 *>(SL + chain * (size_t)D * D + (size_t)(dv0 + 16 * nt + r16) * D +
                                               16 * (W * MPW + a) + 4 * g) = sacc[a][nt];
        }
    };

    // ------------------------------------------------------------------ flow waves
    auto flow_wave = [&](auto Wc, auto Rc) {
        constexpr int W = decltype(Wc)::value;
        constexpr bool kGram = decltype(Rc)::value == 0;           // gram wave (else aux wave)
        const int tb0 = lane0 + 64 * W;                            // thread index among the waves of this role
        int tb = tb0, lane = lane0, r16 = lane & 15, g = lane >> 4;

        constexpr int VPR = D / 8;                                 // 16-byte vectors per row of K
        constexpr int KV = N * D / 8 / NTHR;                       // vectors of K per thread
        constexpr int PPR = TV / 8;                                // 16-byte pieces per row of the V tile
        constexpr int VV = (N * PPR + NTHR - 1) / NTHR;            // vectors of the V tile per thread
        constexpr int OV = (C * PPR + NTHR - 1) / NTHR;            // vectors of the O tile per thread
        constexpr int NT16 = N / 16;

        // ---- who does what among the four flow waves
        // rows (16-row tiles `at`) of the Gram below the diagonal 32-blocks owned by this wave;
        // tile at meets the column tiles bt < 2 (at >> 1)
        constexpr int NOWN = N == 128 ? (W < 2 ? 1 : 2) : (W < 2 ? 1 : 0);
        constexpr auto own_t = [](int i) constexpr {
            if (N == 128) return W == 0 ? 7 : W == 1 ? 6 : W == 2 ? (i == 0 ? 5 : 2) : (i == 0 ? 4 : 3);
            return W == 0 ? 3 : 2;
        };
        // diagonal 32-block built by aux wave W (-1: none)
        constexpr int DB = W < NB ? W : -1;
        // token tiles of P computed by this wave (-1: none)
        constexpr int PT = CT >= 8 ? 2 : 1;
        constexpr auto ptile = [](int i) constexpr {
            if (CT >= 8) {
                const int a = W == 0 ? 7 : W == 1 ? 5 : W == 2 ? 4 : 6;
                return i == 0 ? a : 7 - a;
            }
            return W < CT ? CT - 1 - W : -1;
        };
        // 16-column slices of X = T^T (16 rows of T) owned by this wave in the substitution
        // (N = 128: gram wave W has slice W, aux wave W slice 7 - W, the same amount of work in total
        // per SIMD; N = 64: the gram waves have the four slices)
        constexpr int NS = N / 16;
        constexpr int SLICE = kGram ? W : (NS > 4 ? NS - 1 - W : -1);

        // ---- registers that carry the block in flight (requested right after the previous one went to LDS)
        bf16x8 kreg[KV], vreg[VV], qreg[PT][NKS];   // Q: one set, requested one block ahead (L2 hits: the state waves ask for it earlier)
        bf16 breg;
        bf16x8 pP[PT][NKT];                                        // P of the block last built, until it goes to LDS

        auto fetch_k = [&](size_t cid) {
            const bf16 *Kg = K + cid * (size_t)N * D;
#pragma unroll
            for (int q = 0; q < KV; ++q) kreg[q] = ld8(Kg + (size_t)(tb + NTHR * q) * 8);
            breg = beta[cid * (size_t)N + (tb % N)];
        };
        auto fetch_v = [&](size_t cid) {
            const bf16 *Vg = V + cid * (size_t)N * D + dv0;
#pragma unroll
            for (int q = 0; q < VV; ++q) {
                int v = tb + NTHR * q;
                v = v < N * PPR ? v : N * PPR - 1;                 // clamp instead of branching
                vreg[q] = ld8(Vg + (size_t)(v / PPR) * D + (v % PPR) * 8);
            }
        };
        auto fetch_q = [&](size_t cid) {
            const bf16 *Qc = Q + cid * (size_t)C * D;
#pragma unroll
            for (int i = 0; i < PT; ++i)
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks)
                    if (ptile(i) >= 0) qreg[i][ks] = ld8(Qc + (size_t)(16 * ptile(i) + r16) * D + 32 * ks + 8 * g);
        };
        auto store_k = [&](int slot) {                             // block b goes to LDS slot b & 1
            bf16 *Kd = Ks + slot * N * KP;
#pragma unroll
            for (int q = 0; q < KV; ++q) {
                const int v = tb + NTHR * q;
                st8(&Kd[(v / VPR) * KP + (v % VPR) * 8], kreg[q]);
            }
            if (tb < N) bs[slot * N + tb] = (float)breg;
        };
        auto store_v = [&]() {
#pragma unroll
            for (int q = 0; q < VV; ++q) {
                const int v = tb + NTHR * q;
                if (v < N * PPR) st8(&Vs[(v / PPR) * VP + (v % PPR) * 8], vreg[q]);
            }
        };
        // the O tile of one block (block tokens x TV features), LDS -> its rows of O
        auto copy_out = [&](size_t cid) {
            bf16 *Oc = O + cid * (size_t)C * D;
#pragma unroll
            for (int q = 0; q < OV; ++q) {
                const int v = tb + NTHR * q;
                if ((q + 1) * NTHR <= C * PPR || v < C * PPR)
                    st8(Oc + (size_t)(v / PPR) * D + dv0 + 8 * (v % PPR), ld8(&Ob[(v / PPR) * OP + 8 * (v % PPR)]));
            }
        };
        // P of block cid: registers -> LDS (and, for inspection, to global memory)
        auto dump_p = [&](size_t cid) {
#pragma unroll
            for (int i = 0; i < PT; ++i) {
                const int tt = ptile(i);
                if (tt < 0) continue;
#pragma unroll
                for (int kt = 0; kt < NKT; ++kt)
                    if (kt < p_ksteps(R, tt)) {
                        st8(&Pl[((size_t)p_tile_index(R, tt, kt) * 64 + lane) * 8], pP[i][kt]);
                        if (Pdump && dv0 == 0)
                            st8(Pdump + cid * (size_t)C * N + full_tile_offset(NKT, tt, kt) + lane * 8, pP[i][kt]);
                    }
            }
        };

        // ---- gram waves: the Gram below the diagonal 32-blocks as operand tiles of -G^T (to LDS) and
        // P = Mbar (.) Q K^T (to registers), from the block in K slot S
        auto gram = [&](int slot) {
            const bf16 *Kc = Ks + slot * N * KP;
            const float *bc = bs + slot * N;
            bf16x8 kA[NOWN > 0 ? NOWN : 1][NKS];
            f32x4 nbA[NOWN > 0 ? NOWN : 1];
#pragma unroll
            for (int i = 0; i < NOWN; ++i) {
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) kA[i][ks] = ld8(&Kc[(16 * own_t(i) + r16) * KP + 32 * ks + 8 * g]);
                nbA[i] = -*reinterpret_cast<const f32x4 *>(&bc[16 * own_t(i) + 4 * g]);
            }
            f32x4 pa[PT][2];
#pragma unroll
            for (int bt = 0; bt < NT16; ++bt) {
                bool any = false;
#pragma unroll
                for (int i = 0; i < NOWN; ++i) any = any || (own_t(i) >> 1) > (bt >> 1);
#pragma unroll
                for (int i = 0; i < PT; ++i) any = any || (ptile(i) >= 0 && (bt >> 1) < p_ksteps(R, ptile(i)));
                if (!any) continue;
                bf16x8 kb[NKS];
                int owned = -1;
#pragma unroll
                for (int i = 0; i < NOWN; ++i)
                    if (own_t(i) == bt) owned = i;
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks)
                    kb[ks] = owned >= 0 ? kA[owned >= 0 ? owned : 0][ks] : ld8(&Kc[(16 * bt + r16) * KP + 32 * ks + 8 * g]);
                // off-diagonal Gram: rows a of the owned tile, columns b of tile bt
#pragma unroll
                for (int i = 0; i < NOWN; ++i) {
                    if ((own_t(i) >> 1) > (bt >> 1)) {
                        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ks = 0; ks < NKS; ++ks) acc = mfma16(kA[i][ks], kb[ks], acc);
                        // lane holds -G[a = 16 at + 4 g + e][b = 16 bt + r16]: slots 4 (at & 1) .. + 3 of
                        // the lane's place in operand tile (j = bt >> 1, mi = bt & 1, i = at >> 1)
                        st4(&Gs[((size_t)g_tile_index(NB, bt >> 1, bt & 1, own_t(i) >> 1) * 64 + lane) * 8 + 4 * (own_t(i) & 1)],
                            cvt4(acc * nbA[i]));
                    }
                }
                // P = Mbar (.) Q K^T: rows = the 16 virtual tokens of tile bt, columns = tokens
#pragma unroll
                for (int i = 0; i < PT; ++i) {
                    const int tt = ptile(i);
                    if (tt >= 0 && (bt >> 1) < p_ksteps(R, tt)) {
                        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ks = 0; ks < NKS; ++ks) acc = mfma16(kb[ks], qreg[i][ks], acc);
                        const int t = 16 * tt + r16;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if ((16 * bt + 4 * g + e) / R > t) acc[e] = 0.0f;
                        pa[i][bt & 1] = acc;
                        if (bt & 1) pP[i][bt >> 1] = join(cvt4(pa[i][0]), cvt4(pa[i][1]));
                    }
                }
            }
        };

        // ---- aux waves: diagonal 32-block DB of T (its transpose, as operand tiles, to LDS)
        auto diag = [&](int slot, int mk) {
            if constexpr (DB >= 0) {
                const bf16 *Kc = Ks + slot * N * KP;
                const float *bc = bs + slot * N;
                constexpr int t0 = 2 * DB, t1 = 2 * DB + 1;
                bf16x8 k0[NKS], k1[NKS];
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    k0[ks] = ld8(&Kc[(16 * t0 + r16) * KP + 32 * ks + 8 * g]);
                    k1[ks] = ld8(&Kc[(16 * t1 + r16) * KP + 32 * ks + 8 * g]);
                }
                const f32x4 rb0 = *reinterpret_cast<const f32x4 *>(&bc[16 * t0 + 4 * g]);
                const f32x4 rb1 = *reinterpret_cast<const f32x4 *>(&bc[16 * t1 + 4 * g]);
                const float cb0 = bc[16 * t0 + r16], cb1 = bc[16 * t1 + r16];
                f32x4 x00 = {0.f, 0.f, 0.f, 0.f}, x01 = x00, x11 = x00;
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    x00 = mfma16(k0[ks], k0[ks], x00);   // [a in tile 0][b in tile 0]
                    x01 = mfma16(k0[ks], k1[ks], x01);   // [a in tile 0][b in tile 1]
                    x11 = mfma16(k1[ks], k1[ks], x11);   // [a in tile 1][b in tile 1]
                }
                // M = -N, N = strict-in-time part of diag(beta) K K^T (rows and columns compared
                // by token, i.e. by virtual token >> mask_shift); accumulator tiles of M and M^T
                f32x4 m[2], mt[2], y[2], yt[2], m21t;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int row = 4 * g + e, col = r16;
                    const bool lo = (col >> mask_shift) < (row >> mask_shift);   // column earlier than row
                    const bool up = (row >> mask_shift) < (col >> mask_shift);
                    m[0][e] = lo ? -rb0[e] * x00[e] : 0.0f;
                    mt[0][e] = up ? -cb0 * x00[e] : 0.0f;
                    m[1][e] = lo ? -rb1[e] * x11[e] : 0.0f;
                    mt[1][e] = up ? -cb1 * x11[e] : 0.0f;
                    m21t[e] = -cb1 * x01[e];               // M_21^T[a in tile 0][b in tile 1]
                    const float id = row == col ? 1.0f : 0.0f;
                    y[0][e] = m[0][e] + id; yt[0][e] = mt[0][e] + id;
                    y[1][e] = m[1][e] + id; yt[1][e] = mt[1][e] + id;
                }
                // Y <- Y (Id + M^(2^k)), k = 1, 2, 3 (M is nilpotent of index <= 16)
                const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int k = 0; k < 3; ++k) {
#pragma unroll
                    for (int b2 = 0; b2 < 2; ++b2) {
                        const bf16x4 am = cvt4(mt[b2]), bm = cvt4(m[b2]);   // A(M) = acc(M^T), B(M) = acc(M)
                        const f32x4 m2 = mfma16k(am, bm, z);                 // M M
                        const bf16x4 cyt = cvt4(yt[b2]), cm2 = cvt4(m2);
                        y[b2] = mfma16k(cyt, cm2, y[b2]);                    // Y + Y M2
                        if (k < 2 || b2 == 1) yt[b2] = mfma16k(cm2, cyt, yt[b2]);   // Y^T + M2^T Y^T
                        if (k < 2) mt[b2] = mfma16k(bm, am, z);              // M^T M^T
                        m[b2] = m2;
                    }
                }
                // T_21 = T_22 M_21 T_11
                const f32x4 tmp = mfma16k(cvt4(m21t), cvt4(y[0]), z);
                const f32x4 y21 = mfma16k(cvt4(yt[1]), cvt4(tmp), z);
                bf16x4 z4;
#pragma unroll
                for (int e = 0; e < 4; ++e) z4[e] = (bf16)0.0f;
                st8(&Ts[((size_t)(2 * DB + 0) * 64 + lane) * 8], join(cvt4(y[0]), cvt4(y21)));
                st8(&Ts[((size_t)(2 * DB + 1) * 64 + lane) * 8], join(z4, cvt4(y[1])));
            }
        };

        // ---- block substitution on the transposed system (Proposition 3.3), last block first:
        //      X_j = T_jj^T (E_j - sum_{i > j} G_ij^T X_i),  X = T^T, on this wave's slice of X
        auto subst = [&](size_t cid) {
            if constexpr (SLICE >= 0) {
                constexpr int s = SLICE;                              // columns 16 s .. 16 s + 15 of X
                constexpr int ib = s >> 1;                            // block that holds the slice's diagonal
                bf16x8 X[NB];
#pragma unroll
                for (int step = 0; step < NB; ++step) {
                    const int j = NB - 1 - step;
                    if (ib >= j) {                                    // otherwise X_j is zero on this slice
                        f32x4 acc[2];
#pragma unroll
                        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                acc[mi][e] = (ib == j && (s & 1) == mi && 4 * g + e == r16) ? 1.0f : 0.0f;
#pragma unroll
                        for (int i = 0; i < NB; ++i) {
                            if (i > j && i <= ib) {
#pragma unroll
                                for (int mi = 0; mi < 2; ++mi)
                                    acc[mi] = mfma16(ld8(&Gs[((size_t)g_tile_index(NB, j, mi, i) * 64 + lane) * 8]), X[i], acc[mi]);
                            }
                        }
                        const bf16x8 rb = join(cvt4(acc[0]), cvt4(acc[1]));
                        f32x4 xacc[2];
#pragma unroll
                        for (int mi = 0; mi < 2; ++mi) {
                            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
                            xacc[mi] = mfma16(ld8(&Ts[((size_t)(2 * j + mi) * 64 + lane) * 8]), rb, z);
                        }
                        X[j] = join(cvt4(xacc[0]), cvt4(xacc[1]));
                        // lane (r16, g) holds T[16 s + r16][32 j + kk(g, e)]: the A-operand tile (s, j) as is
                        st8(&Tl[((size_t)t_tile_index(s, j) * 64 + lane) * 8], X[j]);
                        if (Tdump && dv0 == 0)
                            st8(Tdump + cid * (size_t)N * N + full_tile_offset(NKT, s, j) + lane * 8, X[j]);
                    }
                }
            }
        };

        if constexpr (kGram) {
            fetch_q(c0);
        } else {
            fetch_k(c0); fetch_v(c0);
        }

        // Round nb stages block nb and builds its flow while the chain is on block nb - 1.
        auto round = [&](int nb) {
            tb = tb0;
            lane = tb & 63; r16 = lane & 15; g = lane >> 4;
            const bool live = nb < NC;
            const size_t cid = c0 + (live ? nb : NC - 1);
            const size_t nx = nb + 1 < NC ? c0 + nb + 1 : c0 + NC - 1;   // block to request next

            // ---- interval 0 of the chain's block nb - 1
            if constexpr (kGram) {
                if (nb >= 1) dump_p(c0 + nb - 1);
            } else {
                if (nb >= 2) copy_out(c0 + nb - 2);
                if (live) store_k(nb & 1);
                fetch_k(nx);
            }
            __syncthreads();

            // ---- interval 1
            if constexpr (kGram) {
                if (live) gram(nb & 1);
                fetch_q(nx);
            } else {
                if (live) store_v();
                fetch_v(nx);
                if (live) diag(nb & 1, nb - 1);
            }
            __syncthreads();

            // ---- interval 2
            if (live) subst(cid);
            __syncthreads();
        };
        for (int nb = 0; nb <= NC; ++nb) round(nb);
        if constexpr (!kGram) copy_out(c0 + NC - 1);
    };

    constexpr std::integral_constant<int, 0> kRoleGram{};
    constexpr std::integral_constant<int, 1> kRoleAux{};
    switch (wave) {
    case 0: state_wave(std::integral_constant<int, 0>{}); break;
    case 1: state_wave(std::integral_constant<int, 1>{}); break;
    case 2: state_wave(std::integral_constant<int, 2>{}); break;
    case 3: state_wave(std::integral_constant<int, 3>{}); break;
    case 4: flow_wave(std::integral_constant<int, 0>{}, kRoleGram); break;
    case 5: flow_wave(std::integral_constant<int, 1>{}, kRoleGram); break;
    case 6: flow_wave(std::integral_constant<int, 2>{}, kRoleGram); break;
    case 7: flow_wave(std::integral_constant<int, 3>{}, kRoleGram); break;
    case 8: flow_wave(std::integral_constant<int, 0>{}, kRoleAux); break;
    case 9: flow_wave(std::integral_constant<int, 1>{}, kRoleAux); break;
    case 10: flow_wave(std::integral_constant<int, 2>{}, kRoleAux); break;
    default: flow_wave(std::integral_constant<int, 3>{}, kRoleAux); break;
    }
}

// ---------------------------------------------------------------------------- host side
// (d, n, block) with a fused instance; the d_v tile is chosen at launch
#ifndef PF_FUSED_INSTANCES
#define PF_FUSED_INSTANCES(X) \
    X(64, 64, 64) X(64, 64, 32) X(64, 128, 32) X(64, 128, 64) X(64, 128, 128) \
    X(128, 64, 64) X(128, 64, 32) X(128, 128, 32) X(128, 128, 64) X(128, 128, 128)
#endif

bool fused_instance_exists(int d, int n, int chunk)
{
#define X(DD, NN, CC) if (d == DD && n == NN && chunk == CC) return true;
    PF_FUSED_INSTANCES(X)
#undef X
    return false;
}

template <int D, int N, int C, int TV>
static hipError_t launch_fused_tv(const void *Q, const void *K, const void *V, const void *beta, const float *S0,
                                  void *O, float *SL, void *Tdump, void *Pdump, int heads, int NC, int tail,
                                  bool product, hipStream_t stream)
{
    auto kern = fused_kernel<D, N, C, TV>;
    constexpr size_t lds = FusedLds<D, N, C, TV>::total;
    static_assert(lds <= kMaxLdsBytes, "fused kernel LDS plan exceeds the CU");
    int mask_shift = 0;
    if (!product)
        while ((1 << mask_shift) < N / C) ++mask_shift;
    static std::atomic<uint64_t> armed{0};
    hipError_t e = arm_dynamic_lds(armed, reinterpret_cast<const void *>(kern), lds);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)heads * (D / TV);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kFusedThreads), lds, stream, (const bf16 *)Q, (const bf16 *)K,
                       (const bf16 *)V, (const bf16 *)beta, S0, (bf16 *)O, SL, (bf16 *)Tdump, (bf16 *)Pdump,
                       heads, NC, tail, mask_shift);
    return hipGetLastError();
}

// d_v rows per workgroup: 32 when that still gives every compute unit a workgroup and the
// instance fits LDS, else 16.
template <int D, int N, int C>
static constexpr bool fused_wide_fits() { return FusedLds<D, N, C, 32>::total <= kMaxLdsBytes; }

int fused_dv_tile(int heads, int d, int n, int chunk)
{
    bool fits = false;
#define X(DD, NN, CC) if (d == DD && n == NN && chunk == CC) fits = fused_wide_fits<DD, NN, CC>();
    PF_FUSED_INSTANCES(X)
#undef X
    return (fits && (long long)heads * (d / 32) >= (long long)device_cu_count()) ? 32 : 16;
}

hipError_t launch_fused(const void *Q, const void *K, const void *V, const void *beta, const float *S0, void *O,
                        float *SL, void *Tdump, void *Pdump, int heads, int L, int d, int r, int chunk,
                        bool product, hipStream_t stream)
{
    const int NC = L / chunk, tail = L % chunk;   // the tail tokens of every head are skipped
    const int n = chunk * r;
    if (NC == 0) return hipSuccess;
    if ((long long)heads * (d / 16) > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool wide = fused_dv_tile(heads, d, n, chunk) == 32;
#define X(DD, NN, CC)                                                                                          \
    if (d == DD && n == NN && chunk == CC) {                                                                    \
        if constexpr (fused_wide_fits<DD, NN, CC>()) {                                                          \
            if (wide)                                                                                           \
                return launch_fused_tv<DD, NN, CC, 32>(Q, K, V, beta, S0, O, SL, Tdump, Pdump, heads, NC, tail, product, stream); \
        }                                                                                                       \
        return launch_fused_tv<DD, NN, CC, 16>(Q, K, V, beta, S0, O, SL, Tdump, Pdump, heads, NC, tail, product, stream);       \
    }
    PF_FUSED_INSTANCES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace pf
