// State-passing scan fused with the intra-chunk readout: step 3 of Section 3 of ParallelFlow
// (arXiv 2504.00492) as a sequential hand-over of S from chunk to chunk.
//
// Rows of S evolve independently (the recurrence of Section 3.1 multiplies S from the right),
// so a workgroup owns TV rows of S (a tile of d_v) of one (b, h) and walks the chunks.  Per
// chunk, with T = (Id + G)^{-1} and P = Mbar (.) Q K^T from the chunk-flow kernel:
//     R     = beta (.) (V - K S_c^T)      n x TV       (the chunk's values seen from the incoming state)
//     U_eff = T R                         n x TV       (= U' - W S_c^T: U + W S_0^T of Theorem 3.2, sign folded)
//     O_c   = Q S_c^T + P U_eff           chunk x TV   (discrete flow of Section 3.1 cut at each token)
//     S_c+1 = S_c + U_eff^T K             TV x d       (S_1 of Theorem 3.2)
//
// Data movement.  S^T lives in fp32 accumulators (wave w owns d_k rows [w d/4, (w+1) d/4)); a
// bf16 copy in LDS ([d_v][d_k], double buffered) feeds the MFMA operands of the next chunk.
// K, the V tile, Q and beta of a chunk are fetched one chunk ahead into registers with
// coalesced 16-byte loads and staged in LDS at the top of the step; K is read from there both
// row-wise (K S^T) and, through the LDS transposing read, column-wise (K^T U_eff); the V tile is
// read transposed into accumulator layout.  R and U_eff go through LDS once each ([d_v][n]:
// accumulator tiles are 4 consecutive tokens of one feature, i.e. 8-byte writes).  T and P
// tiles are used by exactly one wave each and are loaded straight from global memory into MFMA
// operand registers, one contiguous tile per load, one chunk ahead.  O is computed transposed
// (rows = d_v) so that a lane ends up with 4 consecutive features of one token.
//
// Every fetch is unconditional and branch-free (tiles that are not needed re-read a tile that
// is), because a branch around a load makes every later wait assume the shorter queue.  Where
// the register budget allows a fifth wave (n <= 128), the four compute waves issue no global
// stores inside the chunk loop: O tiles go to LDS and the fifth wave copies them out one step
// later.  With only loads in flight, a wave's memory counter retires in order, so waiting for
// one operand set does not also wait for the sets requested after it.  For n = 256 the operand
// sets need more than 256 registers per lane, which only four waves per workgroup leave room
// for; there the compute waves store O themselves.
#include "pf_internal.h"
#include "pf_common.cuh"
#include "pf_layout.h"

namespace pf {

constexpr int kScanComputeWaves = 4;
constexpr int kScanComputeThreads = 64 * kScanComputeWaves;
template <int N> constexpr bool scan_has_writer() { return N <= 128; }
template <int N> constexpr int scan_threads() { return kScanComputeThreads + (scan_has_writer<N>() ? 64 : 0); }

template <int D, int N, int C, int TV>
struct ScanLds {
    static constexpr int KP = D + 8;   // pitch of a row of K / Q
    static constexpr int VP = TV + 8;  // pitch of a row (virtual token) of the V tile
    static constexpr int SP = D + 8;   // pitch of a row of the bf16 state copy
    static constexpr int UP = N + 8;   // pitch of a row of R^T / U_eff^T
    static constexpr int OP = TV + 8;  // pitch of a row (one token) of the staged O tile
    static constexpr size_t oKs = 0;
    static constexpr size_t oVs = oKs + (size_t)N * KP * 2;
    static constexpr size_t oQs = oVs + (size_t)N * VP * 2;
    static constexpr size_t oBs = oQs + (size_t)C * KP * 2;
    static constexpr size_t oSb = oBs + (size_t)N * 4;
    static constexpr size_t oRs = oSb + (size_t)2 * TV * SP * 2;
    static constexpr size_t oUe = oRs + (size_t)TV * UP * 2;
    static constexpr size_t oOb = oUe + (size_t)TV * UP * 2;
    static constexpr size_t total = oOb + (scan_has_writer<N>() ? (size_t)2 * C * OP * 2 : 0);
};

template <int D, int N, int C, int TV>
__global__ __launch_bounds__(scan_threads<N>()) void scan_kernel(
    const bf16 *__restrict__ Q, const bf16 *__restrict__ K, const bf16 *__restrict__ V,
    const bf16 *__restrict__ beta, const bf16 *__restrict__ Tt, const bf16 *__restrict__ Pt,
    const float *S0, bf16 *__restrict__ O, float *SL, int nchains, int NC)
{
    using Ld = ScanLds<D, N, C, TV>;
    constexpr int R = N / C;
    constexpr int NKS = D / 32;        // k-steps over d
    constexpr int NKT = N / 32;        // k-steps over the chunk's virtual tokens
    constexpr int NNT = TV / 16;       // 16-wide tiles over this workgroup's d_v rows
    constexpr int MT = N / 16;         // 16-row tiles of virtual tokens
    constexpr int CT = C / 16;         // 16-row tiles of tokens
    constexpr int MPW = D / 64;        // d_k tiles (16 rows of S^T) owned by one wave
    constexpr int M1 = MT / 4;         // 16-row tiles of R / U_eff per wave
    constexpr int T2 = CT / 4;         // 16-token tiles of O per wave
    constexpr int KP = Ld::KP, VP = Ld::VP, SP = Ld::SP, UP = Ld::UP, OP = Ld::OP;
    constexpr int NTHR = kScanComputeThreads;
    constexpr bool kWriter = scan_has_writer<N>();
    static_assert(D % 64 == 0 && TV % 16 == 0 && N % 32 == 0, "tile shapes");
    static_assert(MT % 4 == 0 && CT % 4 == 0, "every compute wave owns the same number of tiles");

    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16 *Ks = reinterpret_cast<bf16 *>(smem + Ld::oKs);
    bf16 *Vs = reinterpret_cast<bf16 *>(smem + Ld::oVs);
    bf16 *Qs = reinterpret_cast<bf16 *>(smem + Ld::oQs);
    float *bs = reinterpret_cast<float *>(smem + Ld::oBs);
    bf16 *Sb = reinterpret_cast<bf16 *>(smem + Ld::oSb);
    bf16 *Rs = reinterpret_cast<bf16 *>(smem + Ld::oRs);
    bf16 *Ue = reinterpret_cast<bf16 *>(smem + Ld::oUe);
    bf16 *Ob = reinterpret_cast<bf16 *>(smem + Ld::oOb);

    const int tid0 = threadIdx.x;
    int tid = tid0;
    int w = tid >> 6, lane = tid & 63;
    int r16 = lane & 15, g = lane >> 4;

    // Workgroups of one (b, h) are nchains apart in blockIdx, hence on the same XCD (block ids
    // go round-robin over the 8 XCDs) and share that XCD's L2 for K, Q, T and P, which they all read.
    const int tile = blockIdx.x / nchains;
    const size_t chain = blockIdx.x % nchains;
    const int dv0 = tile * TV;

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

    // ---- register sets that carry the next chunk's operands
    constexpr int VPR = D / 8;                                 // 16-byte vectors per row of K / Q
    constexpr int KV = (N * D / 8 + NTHR - 1) / NTHR;          // vectors of K per thread
    constexpr int QV = (C * D / 8 + NTHR - 1) / NTHR;          // vectors of Q per thread
    constexpr int PPR = TV / 8;                                // 16-byte pieces per row of the V tile
    constexpr int VV = (N * PPR + NTHR - 1) / NTHR;            // vectors of the V tile per thread
    bf16x8 kreg[KV], qreg[QV], vreg[VV];
    bf16 breg = (bf16)0.0f;
    bf16x8 t1[M1][NKT];        // T tiles of this wave's rows of U_eff
    bf16x8 p2[T2][NKT];        // P tiles of this wave's token tiles
    static_assert(N <= NTHR, "beta of a chunk is fetched by one pass");

    // rows of U_eff owned by this wave: tiles w and 7 - w of every group of 8 (evens out the
    // triangular amount of work of T R); one tile per wave when there are only 4
    auto row_tile = [&](int i) { return MT >= 8 ? ((i & 1) ? 8 * (i >> 1) + 7 - w : 8 * (i >> 1) + w) : w + 4 * i; };
    // token tiles of O owned by this wave: w and (with 8 tiles) 7 - w
    auto tok_tile = [&](int i) { return CT >= 8 ? ((i & 1) ? 8 * (i >> 1) + 7 - w : 8 * (i >> 1) + w) : w + 4 * i; };

    auto fetch_in = [&](size_t cid) {
        const bf16 *Kg = K + cid * (size_t)N * D;
        const bf16 *Vg = V + cid * (size_t)N * D + dv0;
        const bf16 *Qg = Q + cid * (size_t)C * D;
#pragma unroll
        for (int q = 0; q < KV; ++q) {
            const int v = tid + NTHR * q;
            if ((q + 1) * NTHR <= N * D / 8 || v < N * D / 8) kreg[q] = ld8(Kg + (size_t)v * 8);
        }
#pragma unroll
        for (int q = 0; q < VV; ++q) {
            int v = tid + NTHR * q;
            v = v < N * PPR ? v : N * PPR - 1;                 // clamp instead of branching
            vreg[q] = ld8(Vg + (size_t)(v / PPR) * D + (v % PPR) * 8);
        }
#pragma unroll
        for (int q = 0; q < QV; ++q) {
            const int v = tid + NTHR * q;
            if ((q + 1) * NTHR <= C * D / 8 || v < C * D / 8) qreg[q] = ld8(Qg + (size_t)v * 8);
        }
        breg = beta[cid * (size_t)N + (tid % N)];
    };
    auto fetch_t = [&](size_t cid) {
        const bf16 *Tc = Tt + cid * (size_t)N * N;
#pragma unroll
        for (int i = 0; i < M1; ++i) {
            const int mt = row_tile(i);
#pragma unroll
            for (int kt = 0; kt < NKT; ++kt) {
                const int kk = 2 * kt <= mt ? kt : 0;          // tiles above the diagonal do not exist
                t1[i][kt] = ld8(Tc + ((size_t)(mt * NKT + kk) * 64 + lane) * 8);
            }
        }
    };
    auto fetch_p = [&](size_t cid) {
        const bf16 *Pc = Pt + cid * (size_t)C * N;
#pragma unroll
        for (int i = 0; i < T2; ++i) {
            const int tt = tok_tile(i);
            const int ksteps = (R * (16 * tt + 16) + 31) / 32;  // causal: virtual tokens < R (16 tt + 16)
#pragma unroll
            for (int kt = 0; kt < NKT; ++kt) {
                const int kk = kt < ksteps ? kt : 0;
                p2[i][kt] = ld8(Pc + ((size_t)(tt * NKT + kk) * 64 + lane) * 8);
            }
        }
    };

    if (NC > 0) {
        fetch_in(chain * (size_t)NC);
        fetch_t(chain * (size_t)NC);
        fetch_p(chain * (size_t)NC);
    }

    for (int ch = 0; ch < NC; ++ch) {
        // The thread id is laundered once per step so that the per-lane LDS and tile offsets of
        // the unrolled code below are recomputed where they are used instead of being hoisted
        // out of this loop and held in registers for the whole kernel.
        tid = tid0;
        asm volatile("" : "+v"(tid));
        w = tid >> 6; lane = tid & 63; r16 = lane & 15; g = lane >> 4;
        const int cur = ch & 1;
        const size_t cid = chain * (size_t)NC + ch;
        const size_t nx = ch + 1 < NC ? cid + 1 : cid;   // last step re-fetches its own chunk
        bf16 *Ocur = Ob + cur * C * OP;
        bf16 *Oc = O + cid * (size_t)C * D;
        const bf16 *Scur = Sb + cur * TV * SP;

        // ---- (0) this chunk's K, V tile, Q, beta: registers -> LDS; next chunk's on their way
#pragma unroll
        for (int q = 0; q < KV; ++q) {
            const int v = tid + NTHR * q;
            if ((q + 1) * NTHR <= N * D / 8 || v < N * D / 8) st8(&Ks[(v / VPR) * KP + (v % VPR) * 8], kreg[q]);
        }
#pragma unroll
        for (int q = 0; q < VV; ++q) {
            const int v = tid + NTHR * q;
            if (v < N * PPR) st8(&Vs[(v / PPR) * VP + (v % PPR) * 8], vreg[q]);
        }
#pragma unroll
        for (int q = 0; q < QV; ++q) {
            const int v = tid + NTHR * q;
            if ((q + 1) * NTHR <= C * D / 8 || v < C * D / 8) st8(&Qs[(v / VPR) * KP + (v % VPR) * 8], qreg[q]);
        }
        if (tid < N) bs[tid] = (float)breg;
        fetch_in(nx);
        __syncthreads();

        // ---- (1a) R = beta (.) (V - K S^T): rows (virtual tokens) dealt to the waves
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
                for (int nt = 0; nt < NNT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    bf16x8 a = ld8(&Ks[(16 * mt + r16) * KP + 32 * ks + 8 * g]);
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt) acc[nt] = mfma16(a, bS[nt][ks], acc[nt]);
                }
                f32x4 bt;
#pragma unroll
                for (int e = 0; e < 4; ++e) bt[e] = bs[16 * mt + 4 * g + e];
#pragma unroll
                for (int nt = 0; nt < NNT; ++nt) {
                    // V tile read transposed: 4 consecutive tokens of feature 16 nt + r16
                    bf16x4 v = lds_read_tr4(&Vs[(16 * mt + 4 * g + (r16 >> 2)) * VP + 16 * nt + 4 * (r16 & 3)]);
                    f32x4 rr = (__builtin_convertvector(v, f32x4) - acc[nt]) * bt;
                    st4(&Rs[(16 * nt + r16) * UP + 16 * mt + 4 * g], cvt4(rr));
                }
            }
        }
        __syncthreads();

        // ---- (1b) U_eff = T R: lower block-triangular, rows dealt so that the waves do equal work
#pragma unroll
        for (int i = 0; i < M1; ++i) {
            const int mt = row_tile(i);
            f32x4 acc[NNT];
#pragma unroll
            for (int nt = 0; nt < NNT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kt = 0; kt < NKT; ++kt) {
                if (2 * kt <= mt) {
#pragma unroll
                    for (int nt = 0; nt < NNT; ++nt)
                        acc[nt] = mfma16(t1[i][kt],
                                         join(ld4(&Rs[(16 * nt + r16) * UP + 32 * kt + 4 * g]),
                                              ld4(&Rs[(16 * nt + r16) * UP + 32 * kt + 16 + 4 * g])),
                                         acc[nt]);
                }
            }
#pragma unroll
            for (int nt = 0; nt < NNT; ++nt) st4(&Ue[(16 * nt + r16) * UP + 16 * mt + 4 * g], cvt4(acc[nt]));
        }
        fetch_t(nx);
        __syncthreads();

        // ---- (2) O^T = S Q^T + U_eff^T P^T : token tiles dealt to the waves
#pragma unroll
        for (int i = 0; i < T2; ++i) {
            const int tt = tok_tile(i);
            f32x4 oacc[NNT];
#pragma unroll
            for (int md = 0; md < NNT; ++md) oacc[md] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                bf16x8 b = ld8(&Qs[(16 * tt + r16) * KP + 32 * ks + 8 * g]);
#pragma unroll
                for (int md = 0; md < NNT; ++md)
                    oacc[md] = mfma16(ld8(&Scur[(16 * md + r16) * SP + 32 * ks + 8 * g]), b, oacc[md]);
            }
            const int ksteps = (R * (16 * tt + 16) + 31) / 32;
#pragma unroll
            for (int kt = 0; kt < NKT; ++kt)
                if (kt < ksteps) {
#pragma unroll
                    for (int md = 0; md < NNT; ++md)
                        oacc[md] = mfma16(join(ld4(&Ue[(16 * md + r16) * UP + 32 * kt + 4 * g]),
                                               ld4(&Ue[(16 * md + r16) * UP + 32 * kt + 16 + 4 * g])),
                                          p2[i][kt], oacc[md]);
                }
#pragma unroll
            for (int md = 0; md < NNT; ++md) {
                if (kWriter) st4(&Ocur[(16 * tt + r16) * OP + 16 * md + 4 * g], cvt4(oacc[md]));
                else st4(Oc + (size_t)(16 * tt + r16) * D + dv0 + 16 * md + 4 * g, cvt4(oacc[md]));
            }
        }
        fetch_p(nx);

        // ---- (3) S^T += K^T U_eff : this wave's d_k rows; K^T comes out of the transposing read
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt) {
            bf16x8 b[NNT];
#pragma unroll
            for (int nt = 0; nt < NNT; ++nt) b[nt] = ld8(&Ue[(16 * nt + r16) * UP + 32 * kt + 8 * g]);
#pragma unroll
            for (int a = 0; a < MPW; ++a) {
                const bf16 *p = &Ks[(32 * kt + 8 * g + (r16 >> 2)) * KP + 16 * (w * MPW + a) + 4 * (r16 & 3)];
                bf16x8 ak = join(lds_read_tr4(p), lds_read_tr4(p + 4 * KP));
#pragma unroll
                for (int nt = 0; nt < NNT; ++nt) sacc[a][nt] = mfma16(ak, b[nt], sacc[a][nt]);
            }
        }
        bf16 *Snext = Sb + (cur ^ 1) * TV * SP;
#pragma unroll
        for (int a = 0; a < MPW; ++a)
#pragma unroll
            for (int nt = 0; nt < NNT; ++nt)
                st4(&Snext[(16 * nt + r16) * SP + 16 * (w * MPW + a) + 4 * g], cvt4(sacc[a][nt]));
        __syncthreads();
    }

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
static hipError_t launch_scan_instance(const void *Q, const void *K, const void *V, const void *beta,
                                       const void *Tt, const void *Pt, const float *S0, void *O, float *SL,
                                       int heads, int NC, hipStream_t stream)
{
    auto kern = scan_kernel<D, N, C, TV>;
    constexpr size_t lds = ScanLds<D, N, C, TV>::total;
    static_assert(lds <= kMaxLdsBytes, "scan kernel LDS plan exceeds the CU");
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)heads * (D / TV);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(scan_threads<N>()), lds, stream, (const bf16 *)Q,
                       (const bf16 *)K, (const bf16 *)V, (const bf16 *)beta, (const bf16 *)Tt,
                       (const bf16 *)Pt, S0, (bf16 *)O, SL, heads, NC);
    return hipGetLastError();
}

hipError_t launch_chunk_scan(const void *Q, const void *K, const void *V, const void *beta, const void *Tt,
                             const void *Pt, const float *S0, void *O, float *SL, int heads, int L, int d,
                             int r, int chunk, hipStream_t stream)
{
    const int NC = L / chunk;
    const int n = chunk * r;
    if ((long long)heads * (d / 16) > 0x7fffffffLL) return hipErrorInvalidValue;
    // d_v tile per workgroup: 32 rows when that already gives at least one workgroup per CU,
    // else 16 rows (twice the workgroups, half the MFMA work per operand byte).  With n = 256
    // only the 16-row tile fits LDS next to the chunk's K.
    const bool wide = (long long)heads * (d / 32) >= 256;
#define X(DD, NN, CC)                                                                                      \
    if (d == DD && n == NN && chunk == CC) {                                                                \
        if constexpr (NN < 256) {                                                                           \
            if (wide)                                                                                       \
                return launch_scan_instance<DD, NN, CC, 32>(Q, K, V, beta, Tt, Pt, S0, O, SL, heads, NC, stream); \
        }                                                                                                   \
        return launch_scan_instance<DD, NN, CC, 16>(Q, K, V, beta, Tt, Pt, S0, O, SL, heads, NC, stream);   \
    }
    PF_SCAN_INSTANCES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace pf
