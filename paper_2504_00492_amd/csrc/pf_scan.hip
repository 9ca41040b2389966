// State-passing scan fused with the intra-chunk readout: step 3 of Section 3 of ParallelFlow
// (arXiv 2504.00492) as a sequential hand-over of S from chunk to chunk.
//
// Rows of S evolve independently (the recurrence of Section 3.1 multiplies S from the right),
// so a workgroup owns TV rows of S (a tile of d_v) of one (b, h) and walks the chunks:
//     U_eff = U' - W S_c^T            n x TV      (U + W S_0^T of Theorem 3.2, sign folded)
//     O_c   = Q S_c^T + P U_eff       chunk x TV  (discrete flow of Section 3.1 cut at each t)
//     S_c+1 = S_c + U_eff^T K         TV x d      (S_1 of Theorem 3.2)
// with W, U', K^T, P and Q as written by the chunk-flow kernel (tiled operand arrays, see
// pf_layout.h).
//
// Data movement.  S^T lives in fp32 accumulators (wave w owns d_k rows [w d/4, (w+1) d/4));
// a bf16 copy in LDS ([d_v][d_k], double buffered) feeds the MFMA operands of the next chunk.
// U_eff goes through LDS once ([d_v][n]: accumulator tiles are 4 consecutive tokens of one
// feature, i.e. 8-byte writes).  W, K^T, Q and P are each used by exactly one wave, so they
// are loaded straight from global memory into MFMA operand registers, one contiguous tile per
// load, one chunk ahead of their use.  O is computed transposed (rows = d_v) so that a lane
// ends up with 4 consecutive features of one token.
//
// Where the register budget allows a fifth wave (n <= 128), the four compute waves issue no
// global stores inside the chunk loop: O tiles go to LDS and the fifth wave copies them out one
// step later.  With only loads in flight, a wave's memory counter retires in order, so waiting
// for one operand set does not also wait for the sets that were requested after it - which is
// what keeps the one-chunk-ahead fetch ahead.  For n = 256 the operand sets need more than 256
// registers per lane, which only four waves per workgroup leave room for; there the compute
// waves store O themselves.
#include "pf_internal.h"
#include "pf_common.cuh"
#include "pf_layout.h"

namespace pf {

constexpr int kScanComputeWaves = 4;
template <int N> constexpr bool scan_has_writer() { return N <= 128; }
template <int N> constexpr int scan_threads() { return 64 * (kScanComputeWaves + (scan_has_writer<N>() ? 1 : 0)); }

template <int D, int N, int C, int TV>
struct ScanLds {
    static constexpr int SP = D + 8;   // pitch of a row of the bf16 state copy
    static constexpr int UP = N + 8;   // pitch of a row of U_eff^T
    static constexpr int OP = TV + 8;  // pitch of a row (one token) of the staged O tile
    static constexpr size_t oSb = 0;
    static constexpr size_t oUe = oSb + (size_t)2 * TV * SP * 2;
    static constexpr size_t oOb = oUe + (size_t)TV * UP * 2;
    static constexpr size_t total = oOb + (scan_has_writer<N>() ? (size_t)2 * C * OP * 2 : 0);
};

template <int D, int N, int C, int TV>
__global__ __launch_bounds__(scan_threads<N>()) void scan_kernel(const bf16 *__restrict__ Wt, const bf16 *__restrict__ Ut,
                                                   const bf16 *__restrict__ Kt, const bf16 *__restrict__ Pt,
                                                   const bf16 *__restrict__ Qt, const float *S0,
                                                   bf16 *__restrict__ O, float *SL, int nchains, int NC)
{
    using Ld = ScanLds<D, N, C, TV>;
    constexpr int R = N / C;
    constexpr int NKS = D / 32;        // k-steps over d
    constexpr int NNT = TV / 16;       // 16-wide tiles over this workgroup's d_v rows
    constexpr int MPW = D / 64;        // d_k tiles (16 rows of S^T) owned by one wave
    constexpr int DT = D / 16;
    constexpr int SP = Ld::SP, UP = Ld::UP, OP = Ld::OP;
    static_assert(D % 64 == 0 && TV % 16 == 0 && N % 32 == 0 && C % 16 == 0, "tile shapes");

    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16 *Sb = reinterpret_cast<bf16 *>(smem + Ld::oSb);
    bf16 *Ue = reinterpret_cast<bf16 *>(smem + Ld::oUe);
    bf16 *Ob = reinterpret_cast<bf16 *>(smem + Ld::oOb);

    const int tid = threadIdx.x;
    const int w = tid >> 6, lane = tid & 63;
    const int r16 = lane & 15, g = lane >> 4;

    // Workgroups of one (b, h) are nchains apart in blockIdx, hence on the same XCD (block ids
    // go round-robin over the 8 XCDs) and share that XCD's L2 for the operands they all read.
    const int tile = blockIdx.x / nchains;
    const size_t chain = blockIdx.x % nchains;
    const int dv0 = tile * TV;

    constexpr bool kWriter = scan_has_writer<N>();
    if (kWriter && w == kScanComputeWaves) {
        // ---- writer wave: after each step's closing barrier, copy that step's O tile
        // (chunk tokens x TV features) from LDS to its rows of O.  It takes part in every
        // barrier of the compute waves and touches nothing else.
        constexpr int PPT = TV / 8;              // 16-byte pieces per token
        constexpr int TPI = 64 / PPT;            // tokens per pass of the wave
        __syncthreads();                         // pairs with the barrier after the initial state
        for (int ch = 0; ch < NC; ++ch) {
            __syncthreads();
            __syncthreads();
            const bf16 *src = Ob + (ch & 1) * C * OP;
            bf16 *Oc = O + (chain * (size_t)NC + ch) * (size_t)C * D;
#pragma unroll
            for (int t0 = 0; t0 < C; t0 += TPI) {
                const int t = t0 + lane / PPT, pc = lane % PPT;
                st8(Oc + (size_t)t * D + dv0 + 8 * pc, ld8(&src[t * OP + 8 * pc]));
            }
        }
        return;
    }

    // ---- initial state: fp32 accumulators + bf16 copy
    f32x4 sacc[MPW][NNT];
#pragma unroll
    for (int a = 0; a < MPW; ++a)
#pragma unroll
        for (int nt = 0; nt < NNT; ++nt) {
            const int mt = w * MPW + a;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (S0) v = *reinterpret_cast<const f32x4 *>(S0 + chain * (size_t)D * D +
                                                         (size_t)(dv0 + 16 * nt + r16) * D + 16 * mt + 4 * g);
            sacc[a][nt] = v;
            st4(&Sb[(16 * nt + r16) * SP + 16 * mt + 4 * g], cvt4(v));
        }
    __syncthreads();

    // Operands that do not depend on the state (W, U', Q, P, K^T of a chunk) are fetched one
    // chunk ahead, straight into the MFMA operand registers: each set is refilled for chunk
    // c+1 right after its last use in chunk c, so the loads fly under the rest of the step.
    constexpr int M1 = N / 64;         // 16-row tiles of U_eff per wave
    constexpr int T2 = (C / 16 + 3) / 4;   // 16-token tiles of O per wave
    constexpr int NKT = N / 32;        // k-steps over the chunk's virtual tokens
    bf16x8 a1[M1][NKS];
    bf16x4 u1[M1][NNT];
    bf16x8 q2[T2][NKS];
    bf16x8 p2[T2][NKT];
    bf16x8 k3[MPW][NKT];

    auto load1 = [&](size_t cid) {
        const bf16 *Wc = Wt + cid * (size_t)N * D;
        const bf16 *Uc = Ut + cid * (size_t)N * D;
#pragma unroll
        for (int i = 0; i < M1; ++i) {
            const int mt = w + 4 * i;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) a1[i][ks] = ld8(Wc + ((size_t)(mt * NKS + ks) * 64 + lane) * 8);
#pragma unroll
            for (int nt = 0; nt < NNT; ++nt) u1[i][nt] = ld4(Uc + ((size_t)(mt * DT + dv0 / 16 + nt) * 64 + lane) * 4);
        }
    };
    static_assert((C / 16) % kScanComputeWaves == 0, "every compute wave owns the same number of token tiles");
    auto load2 = [&](size_t cid) {
        const bf16 *Pc = Pt + cid * (size_t)C * N;
        const bf16 *Qc = Qt + cid * (size_t)C * D;
#pragma unroll
        for (int i = 0; i < T2; ++i) {
            const int tt = w + 4 * i;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) q2[i][ks] = ld8(Qc + ((size_t)(tt * NKS + ks) * 64 + lane) * 8);
            // Tiles behind the causal limit (32 ks >= R (16 tt + 16)) were never written and are
            // never multiplied; their slots re-read tile 0 so that the load sequence has no
            // branch (a branch here would make every later wait a full drain).
            const int ksteps = (R * (16 * tt + 16) + 31) / 32;
#pragma unroll
            for (int ks = 0; ks < NKT; ++ks) {
                const int kk = ks < ksteps ? ks : 0;
                p2[i][ks] = ld8(Pc + ((size_t)(tt * NKT + kk) * 64 + lane) * 8);
            }
        }
    };
    auto load3 = [&](size_t cid) {
        const bf16 *Kc = Kt + cid * (size_t)N * D;
#pragma unroll
        for (int a = 0; a < MPW; ++a)
#pragma unroll
            for (int ks = 0; ks < NKT; ++ks)
                k3[a][ks] = ld8(Kc + ((size_t)((w * MPW + a) * NKT + ks) * 64 + lane) * 8);
    };

    // ---- L2 warm-up.  A workgroup can only keep so many bytes in flight, so at HBM latency the
    // demand loads above would be what bounds a step.  Two steps ahead of its use, every line of
    // a chunk's operand arrays is touched once (one dword per 128-byte line); the tiles of one
    // (b, h) share an L2 and split the lines among themselves, so this costs each wave a couple
    // of load instructions per step and turns the demand loads into L2 hits.  The touched words
    // are never looked at.
    constexpr int kAhead = 2;
    constexpr int NTILES = D / TV;
    constexpr int kLine = 64;                                   // bf16 elements per 128-byte line
    constexpr int LW = (N * D / kLine + NTILES - 1) / NTILES;   // lines of Wt (and of Kt) per tile
    constexpr int LP = (C * N / kLine + NTILES - 1) / NTILES;   // lines of Pt per tile
    constexpr int LQ = (C * D / kLine + NTILES - 1) / NTILES;   // lines of Qt per tile
    constexpr int LU = N * TV / kLine;                          // lines of this tile's part of Ut
    constexpr int LMAX = LW > LP ? (LW > LU ? LW : LU) : (LP > LU ? LP : LU);
    // Measured: it pays for n = 256 (about 8 %), and costs a little for the smaller chunks.
    constexpr bool kWarm = N >= 256;
    constexpr int T0 = kWarm ? (LMAX + 63) / 64 : 0, T1 = kWarm ? (LQ + 63) / 64 : 0, NTOUCH = T0 + T1;
    // wave 0: Wt, wave 1: Kt, wave 2: Pt, wave 3: this tile's Ut and (second job) Qt
    const bf16 *tbase[NTOUCH + 1];
    size_t tstride[NTOUCH + 1];
    if (kWarm) {
        const bf16 *b0 = w == 0 ? Wt : w == 1 ? Kt : w == 2 ? Pt : Ut;
        const size_t st0 = w == 2 ? (size_t)C * N : (size_t)N * D;
        const int total0 = w == 2 ? C * N / kLine : N * D / kLine;
        const int cnt0 = w < 2 ? LW : w == 2 ? LP : LU;
#pragma unroll
        for (int k = 0; k < T0; ++k) {
            int j = lane + 64 * k;
            j = j < cnt0 ? j : cnt0 - 1;
            size_t el;
            if (w == 3) {   // Ut tiles of this d_v tile: [mt][dt][64 lanes][4]; TV*16 elements per mt
                constexpr int per_mt = TV * 16 / kLine > 0 ? TV * 16 / kLine : 1;
                el = (size_t)((j / per_mt) * DT + dv0 / 16) * 256 + (size_t)(j % per_mt) * kLine;
            } else {
                int line = tile * cnt0 + j;
                line = line < total0 ? line : total0 - 1;
                el = (size_t)line * kLine;
            }
            tbase[k] = b0 + chain * (size_t)NC * st0 + el;
            tstride[k] = st0;
        }
#pragma unroll
        for (int k = 0; k < T1; ++k) {
            int j = lane + 64 * k;
            j = j < LQ ? j : LQ - 1;
            int line = tile * LQ + j;
            line = line < C * D / kLine ? line : C * D / kLine - 1;
            // only wave 3 has a second job; the others re-touch their own first line
            tbase[T0 + k] = w == 3 ? Qt + chain * (size_t)NC * C * D + (size_t)line * kLine : tbase[0];
            tstride[T0 + k] = w == 3 ? (size_t)C * D : tstride[0];
        }
    }
    // The touched word is "used" by an empty asm statement one step later, just before the
    // register is reloaded: late enough that the load has long returned, and enough to keep the
    // compiler from dropping it.
    uint32_t touched[NTOUCH + 1];
#pragma unroll
    for (int k = 0; k < NTOUCH; ++k) touched[k] = 0;
    auto touch = [&](int c) {   // c = chunk index within this (b, h)
#pragma unroll
        for (int k = 0; k < NTOUCH; ++k) {
            asm volatile("" ::"v"(touched[k]));
            touched[k] = *reinterpret_cast<const uint32_t *>(tbase[k] + (size_t)c * tstride[k]);
        }
    };

    if (NC > 0) {
        load1(chain * (size_t)NC);
        load2(chain * (size_t)NC);
        load3(chain * (size_t)NC);
    }

    for (int ch = 0; ch < NC; ++ch) {
        const int cur = ch & 1;
        const size_t cid = chain * (size_t)NC + ch;
        // The fetch for "the next chunk" is unconditional (the last step re-fetches its own chunk):
        // a branch around it would force every later wait to assume the shorter queue.
        const size_t nx = ch + 1 < NC ? cid + 1 : cid;
        bf16 *Ocur = Ob + cur * C * OP;
        bf16 *Oc = O + cid * (size_t)C * D;
        const bf16 *Scur = Sb + cur * TV * SP;

        // ---- (1) U_eff = U' + Wneg S^T : rows (virtual tokens) dealt to the waves
        {
            bf16x8 bS[NNT][NKS];
#pragma unroll
            for (int nt = 0; nt < NNT; ++nt)
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) bS[nt][ks] = ld8(&Scur[(16 * nt + r16) * SP + 32 * ks + 8 * g]);
#pragma unroll
            for (int i = 0; i < M1; ++i) {
                const int mt = w + 4 * i;
                f32x4 acc[NNT];
#pragma unroll
                for (int nt = 0; nt < NNT; ++nt) acc[nt] = __builtin_convertvector(u1[i][nt], f32x4);
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt) acc[nt] = mfma16(a1[i][ks], bS[nt][ks], acc[nt]);
#pragma unroll
                for (int nt = 0; nt < NNT; ++nt) st4(&Ue[(16 * nt + r16) * UP + 16 * mt + 4 * g], cvt4(acc[nt]));
            }
        }
        load1(nx);
        __syncthreads();

        // ---- (2) O^T = S Q^T + U_eff^T P^T : token tiles dealt to the waves
#pragma unroll
        for (int i = 0; i < T2; ++i) {
            const int tt = w + 4 * i;
            {
                f32x4 oacc[NNT];
#pragma unroll
                for (int md = 0; md < NNT; ++md) oacc[md] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                    for (int md = 0; md < NNT; ++md)
                        oacc[md] = mfma16(ld8(&Scur[(16 * md + r16) * SP + 32 * ks + 8 * g]), q2[i][ks], oacc[md]);
                const int ksteps = (R * (16 * tt + 16) + 31) / 32;
#pragma unroll
                for (int ks = 0; ks < NKT; ++ks)
                    if (ks < ksteps) {
#pragma unroll
                        for (int md = 0; md < NNT; ++md)
                            oacc[md] = mfma16(join(ld4(&Ue[(16 * md + r16) * UP + 32 * ks + 4 * g]),
                                                   ld4(&Ue[(16 * md + r16) * UP + 32 * ks + 16 + 4 * g])),
                                              p2[i][ks], oacc[md]);
                    }
#pragma unroll
                for (int md = 0; md < NNT; ++md)
                    if (kWriter) st4(&Ocur[(16 * tt + r16) * OP + 16 * md + 4 * g], cvt4(oacc[md]));
                    else st4(Oc + (size_t)(16 * tt + r16) * D + dv0 + 16 * md + 4 * g, cvt4(oacc[md]));
            }
        }
        load2(nx);

        // ---- (3) S^T += K^T U_eff : this wave's d_k rows
#pragma unroll
        for (int ks = 0; ks < NKT; ++ks) {
            bf16x8 b[NNT];
#pragma unroll
            for (int nt = 0; nt < NNT; ++nt) b[nt] = ld8(&Ue[(16 * nt + r16) * UP + 32 * ks + 8 * g]);
#pragma unroll
            for (int a = 0; a < MPW; ++a)
#pragma unroll
                for (int nt = 0; nt < NNT; ++nt) sacc[a][nt] = mfma16(k3[a][ks], b[nt], sacc[a][nt]);
        }
        load3(nx);
        touch(ch + kAhead < NC ? ch + kAhead : ch);
        bf16 *Snext = Sb + (cur ^ 1) * TV * SP;
#pragma unroll
        for (int a = 0; a < MPW; ++a)
#pragma unroll
            for (int nt = 0; nt < NNT; ++nt)
                st4(&Snext[(16 * nt + r16) * SP + 16 * (w * MPW + a) + 4 * g], cvt4(sacc[a][nt]));
        __syncthreads();
    }

#pragma unroll
    for (int k = 0; k < NTOUCH; ++k) asm volatile("" ::"v"(touched[k]));
    if (SL) {
#pragma unroll
        for (int a = 0; a < MPW; ++a)
#pragma unroll
            for (int nt = 0; nt < NNT; ++nt)
                *reinterpret_cast<f32x4 *>(SL + chain * (size_t)D * D + (size_t)(dv0 + 16 * nt + r16) * D +
                                           16 * (w * MPW + a) + 4 * g) = sacc[a][nt];
    }
}

// ---------------------------------------------------------------------------- host side
#define PF_SCAN_INSTANCES(X) \
    X(64, 64, 64) X(64, 128, 64) X(64, 128, 128) X(64, 256, 64) X(64, 256, 128) \
    X(128, 64, 64) X(128, 128, 64) X(128, 128, 128) X(128, 256, 64) X(128, 256, 128)

template <int D, int N, int C, int TV>
static hipError_t launch_scan_instance(const void *Wt, const void *Ut, const void *Kt, const void *Pt,
                                       const void *Qt, const float *S0, void *O, float *SL, int heads,
                                       int NC, hipStream_t stream)
{
    auto kern = scan_kernel<D, N, C, TV>;
    constexpr size_t lds = ScanLds<D, N, C, TV>::total;
    static_assert(lds <= 64 * 1024, "scan kernel is meant to leave room for several workgroups per CU");
    const unsigned grid = (unsigned)heads * (D / TV);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(scan_threads<N>()), lds, stream, (const bf16 *)Wt, (const bf16 *)Ut,
                       (const bf16 *)Kt, (const bf16 *)Pt, (const bf16 *)Qt, S0, (bf16 *)O, SL, heads, NC);
    return hipGetLastError();
}

hipError_t launch_chunk_scan(const void *Wt, const void *Ut, const void *Kt, const void *Pt,
                             const void *Qt, const float *S0, void *O, float *SL, int heads, int L, int d,
                             int r, int chunk, hipStream_t stream)
{
    const int NC = L / chunk;
    const int n = chunk * r;
    if ((long long)heads * (d / 16) > 0x7fffffffLL) return hipErrorInvalidValue;
    // d_v tile per workgroup: 32 rows when that already gives at least one workgroup per CU,
    // else 16 rows (twice the workgroups, half the MFMA work per operand byte).
    const bool wide = (long long)heads * (d / 32) >= 256;
#define X(DD, NN, CC)                                                                                   \
    if (d == DD && n == NN && chunk == CC)                                                               \
        return wide ? launch_scan_instance<DD, NN, CC, 32>(Wt, Ut, Kt, Pt, Qt, S0, O, SL, heads, NC, stream) \
                    : launch_scan_instance<DD, NN, CC, 16>(Wt, Ut, Kt, Pt, Qt, S0, O, SL, heads, NC, stream);
    PF_SCAN_INSTANCES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace pf
