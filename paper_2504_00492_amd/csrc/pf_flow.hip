// Chunk-flow kernel: step 2 of Section 3 of ParallelFlow (arXiv 2504.00492), "parallel
// compute".  One workgroup (8 wavefronts) per (b, h, chunk); no dependence between chunks.
//
// In delta variables (Remark in Section 3.1: A = beta k, Atil = -beta v, B = -k) Theorem 3.2
// reads, with n = chunk * r virtual tokens and M strict in time,
//     (Id + G) W = beta (.) K,   (Id + G) U' = beta (.) V,   G = M (.) diag(beta) K K^T,
// where U' = -U.  The system is solved by block forward substitution (Proposition 3.3) on
// 32-row blocks, directly for the right-hand sides (the n x n inverse is never formed):
//     X_i = T_ii ( beta_i (.) [K_i | V_i]  -  sum_{j<i} G_ij X_j ),    T_ii = (Id + G_ii)^{-1}.
// T_ii (32 x 32) comes from two 16 x 16 forward substitutions in fp32 on the vector ALU and
// one block merge  T_21 = -T_22 G_21 T_11  on MFMA.
//
// Work split.  The 2 d right-hand-side columns are dealt to the 8 wavefronts (waves 0-3 the
// key columns, waves 4-7 the value columns).  A wave keeps every finished X_j of its column
// slice in registers, already in MFMA B-operand form, so the substitution itself needs no
// LDS traffic for X.  G_ij and T_ii are built cooperatively and read by all waves as A
// operands from LDS.  Gram blocks are computed transposed so that an accumulator tile (4
// consecutive j per lane) goes to row-major LDS with 8-byte writes.
//
// The kernel is persistent: a workgroup walks chunks blockIdx.x, blockIdx.x + gridDim.x, ...
// and, while it works on one chunk, the K, V, beta and Q of its next chunk are already on
// their way from HBM into registers (each register set is refilled right after its last use),
// so that loads and MFMA work of neighbouring chunks overlap on a CU that, because of the LDS
// footprint, holds a single workgroup.
//
// Outputs: the tiled operand arrays described in pf_layout.h.
#include "pf_internal.h"
#include "pf_common.cuh"
#include "pf_layout.h"

namespace pf {

constexpr int kFlowThreads = 512;
constexpr int kFlowWaves = kFlowThreads / 64;

template <int D, int N, int C>
struct FlowLds {
    static constexpr int NB = N / 32;       // 32-row blocks per chunk
    static constexpr int KP = D + 8;        // pitch of K / V / Q rows (bf16)
    static constexpr int GP = N + 8;        // pitch of a G block-row (bf16)
    static constexpr int TP = 40;           // pitch of a T_ii row (bf16)
    static constexpr int NP = 36;           // pitch of the fp32 scratch used to build T_ii
    static constexpr int FW = D / 4;        // right-hand-side columns per wave
    static constexpr int WP = FW + 8;       // pitch of the per-wave W staging tile (bf16)
    static constexpr size_t oKs = 0;
    static constexpr size_t oBs = oKs + (size_t)N * KP * 2;
    static constexpr size_t oTs = oBs + (size_t)N * 4;
    static constexpr size_t oUn = oTs + (size_t)NB * 32 * TP * 2;       // region reused by phase
    // phase "build T": fp32 scratch, one 32 x NP tile per wave that has a diagonal block
    static constexpr size_t szNs = (size_t)(NB < kFlowWaves ? NB : kFlowWaves) * 32 * NP * 4;
    // phase "substitute": G block-row (x2), W staging (4 waves), V block (x2).  The V buffers
    // lie behind the scratch tiles because V block 0 is staged before T is built.
    static constexpr size_t oGs = oUn;
    static constexpr size_t oWs = oGs + (size_t)2 * 32 * GP * 2;
    static constexpr size_t oVs = oWs + (size_t)4 * 32 * WP * 2;
    static_assert(oVs - oUn >= szNs, "V buffers must not overlap the scratch tiles");
    static constexpr size_t szS = oVs + (size_t)2 * 32 * KP * 2 - oUn;
    // phase "P": the chunk's queries
    static constexpr size_t szQ = (size_t)C * KP * 2;
    static constexpr size_t szUn = szNs > szS ? (szNs > szQ ? szNs : szQ) : (szS > szQ ? szS : szQ);
    static constexpr size_t total = oUn + szUn;
};

template <int D, int N, int C>
__global__ __launch_bounds__(kFlowThreads) void flow_kernel(
    const bf16 *__restrict__ Q, const bf16 *__restrict__ K, const bf16 *__restrict__ V,
    const bf16 *__restrict__ beta, bf16 *__restrict__ Wt, bf16 *__restrict__ Ut, bf16 *__restrict__ Kt,
    bf16 *__restrict__ Pt, bf16 *__restrict__ Qt, int nchunks)
{
    using Ld = FlowLds<D, N, C>;
    constexpr int R = N / C;          // rank: virtual tokens per token
    constexpr int NB = Ld::NB;
    constexpr int FW = Ld::FW;
    constexpr int NT = FW / 16;       // 16-column tiles of the right-hand side per wave
    constexpr int NKS = D / 32, NKT = N / 32, DT = D / 16, CT = C / 16;
    constexpr int KP = Ld::KP, GP = Ld::GP, TP = Ld::TP, NP = Ld::NP, WP = Ld::WP;
    constexpr int NTHR = kFlowThreads;
    static_assert(32 % R == 0 && N % 32 == 0 && C % 16 == 0 && D % 64 == 0, "tile shapes");

    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16 *Ks = reinterpret_cast<bf16 *>(smem + Ld::oKs);
    float *bs = reinterpret_cast<float *>(smem + Ld::oBs);
    bf16 *Ts = reinterpret_cast<bf16 *>(smem + Ld::oTs);
    float *NsAll = reinterpret_cast<float *>(smem + Ld::oUn);
    bf16 *Vs = reinterpret_cast<bf16 *>(smem + Ld::oVs);
    bf16 *Gs = reinterpret_cast<bf16 *>(smem + Ld::oGs);
    bf16 *WsAll = reinterpret_cast<bf16 *>(smem + Ld::oWs);
    bf16 *Qs = reinterpret_cast<bf16 *>(smem + Ld::oUn);

    const int tid0 = threadIdx.x;

    // ---- register sets that carry the next chunk's inputs
    constexpr int VPR = D / 8;                         // 16-byte vectors per row
    constexpr int KV = (N * D / 8 + NTHR - 1) / NTHR;  // vectors of K (and of V) per thread
    constexpr int QV = (C * D / 8 + NTHR - 1) / NTHR;  // vectors of Q per thread
    constexpr int VVEC = 32 * VPR;                     // vectors in one 32-row block
    constexpr int BPP = NTHR / VVEC;                   // 32-row blocks covered by one pass of the workgroup
    static_assert(VVEC <= NTHR && NTHR % VVEC == 0, "a pass covers whole blocks");
    constexpr int VR = KV > 4 ? 4 : KV;                // V travels through a ring of VR passes
    static_assert(KV % VR == 0, "ring slots are reused with a fixed stride");
    bf16x8 kreg[KV], vreg[VR], qreg[QV];
    bf16 breg = (bf16)0.0f;   // kept as loaded: converting here would wait for the fetch

    auto fetch_k = [&](size_t c) {
        const bf16 *Kg = K + c * (size_t)N * D;
#pragma unroll
        for (int q = 0; q < KV; ++q) {
            const int v = tid0 + NTHR * q;
            if ((q + 1) * NTHR <= N * D / 8 || v < N * D / 8) kreg[q] = ld8(Kg + (size_t)v * 8);
        }
        breg = beta[c * (size_t)N + (tid0 % N)];   // every thread loads: no branch, always in range
    };
    auto fetch_v_pass = [&](size_t c, int q) {       // the blocks [q BPP, (q+1) BPP) of V
        const int v = tid0 + NTHR * q;
        if ((q + 1) * NTHR <= N * D / 8 || v < N * D / 8) vreg[q % VR] = ld8(V + c * (size_t)N * D + (size_t)v * 8);
    };
    auto fetch_q = [&](size_t c) {
        const bf16 *Qg = Q + c * (size_t)C * D;
#pragma unroll
        for (int q = 0; q < QV; ++q) {
            const int v = tid0 + NTHR * q;
            if ((q + 1) * NTHR <= C * D / 8 || v < C * D / 8) qreg[q] = ld8(Qg + (size_t)v * 8);
        }
    };
    static_assert(N <= NTHR, "beta of a chunk is fetched by one pass");

    size_t cid = blockIdx.x;
    if (cid < (size_t)nchunks) {
        fetch_k(cid);
#pragma unroll
        for (int q = 0; q < VR; ++q) fetch_v_pass(cid, q);
        fetch_q(cid);
    }

    for (; cid < (size_t)nchunks; cid += gridDim.x) {
        // The thread id is laundered once per chunk so that the many per-lane LDS offsets of the
        // unrolled code below are recomputed where they are used instead of being hoisted out
        // of this loop and held in registers for the whole kernel.
        int tid = tid0;
        asm volatile("" : "+v"(tid));
        const int w = tid >> 6, lane = tid & 63;
        const int r16 = lane & 15, g = lane >> 4;
        const bool isV = w >= 4;               // waves 4-7 solve for U', waves 0-3 for W
        const int cb = (w & 3) * FW;           // first column of this wave's slice inside K or V

        const size_t nxt = cid + gridDim.x;
        const bool more = nxt < (size_t)nchunks;
        bf16 *Wg = Wt + cid * (size_t)N * D;
        bf16 *Ug = Ut + cid * (size_t)N * D;
        bf16 *Ktg = Kt + cid * (size_t)N * D;
        bf16 *Ptg = Pt + cid * (size_t)C * N;
        bf16 *Qtg = Qt + cid * (size_t)C * D;

        // ------------------------------------------------------------ K, beta: registers -> LDS
#pragma unroll
        for (int q = 0; q < KV; ++q) {
            const int v = tid + NTHR * q;
            if ((q + 1) * NTHR <= N * D / 8 || v < N * D / 8) st8(&Ks[(v / VPR) * KP + (v % VPR) * 8], kreg[q]);
        }
        if (tid < N) bs[tid] = (float)breg;
        // V block b: registers -> LDS buffer (b & 1).  When that frees a ring slot, the slot is
        // refilled with the pass VR further down the stream (this chunk's, then the next one's).
        auto stage_v = [&](int b) {
            const int q = b / BPP;
            if (tid / VVEC == b % BPP)
                st8(&Vs[(b & 1) * 32 * KP + ((tid % VVEC) / VPR) * KP + (tid % VPR) * 8], vreg[q % VR]);
            if (b % BPP == BPP - 1 || b == NB - 1) {
                if (q + VR < KV) fetch_v_pass(cid, q + VR);
                else if (more) fetch_v_pass(nxt, q + VR - KV);
            }
        };
        stage_v(0);
        __syncthreads();
        if (more) fetch_k(nxt);

        // ------------------------------------------------------------ K^T tiles out
        for (int it = w; it < DT * NKT; it += kFlowWaves) {
            const int a = it / NKT, kt = it % NKT;
            const bf16 *p = &Ks[(32 * kt + 8 * g + (r16 >> 2)) * KP + 16 * a + 4 * (r16 & 3)];
            bf16x4 lo = lds_read_tr4(p), hi = lds_read_tr4(p + 4 * KP);
            st8(Ktg + ((size_t)(a * NKT + kt) * 64 + lane) * 8, join(lo, hi));
        }

        // ------------------------------------------------------------ T_ii for every 32-block
        // Each wave builds whole diagonal blocks on its own (private scratch tile, private
        // destination), so the steps below are ordered by program order within the wave.
        {
            float *Ns = NsAll + w * 32 * NP;
            for (int db = w; db < NB; db += kFlowWaves) {
                // N_db = strict-in-time part of diag(beta) K K^T on the block, fp32, row-major
                f32x4 acc[3];
#pragma unroll
                for (int t3 = 0; t3 < 3; ++t3) acc[t3] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    bf16x8 k0 = ld8(&Ks[(32 * db + r16) * KP + 32 * ks + 8 * g]);
                    bf16x8 k1 = ld8(&Ks[(32 * db + 16 + r16) * KP + 32 * ks + 8 * g]);
                    acc[0] = mfma16(k0, k0, acc[0]);   // rows 0-15,  cols 0-15
                    acc[1] = mfma16(k1, k0, acc[1]);   // rows 16-31, cols 0-15
                    acc[2] = mfma16(k1, k1, acc[2]);   // rows 16-31, cols 16-31
                }
#pragma unroll
                for (int tile = 0; tile < 4; ++tile) {
                    const int mi = tile >> 1, ni = tile & 1;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const int row = 16 * mi + 4 * g + jj, col = 16 * ni + r16;
                        float val = 0.0f;
                        if (tile != 1 && (col / R < row / R))
                            val = acc[tile == 0 ? 0 : tile - 1][jj] * bs[32 * db + row];
                        Ns[row * NP + col] = val;
                    }
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                if (lane < 32) {
                    // two 16 x 16 unit-lower-triangular inverses, lane = (sub-block, column)
                    const int o = 16 * (lane >> 4), c = lane & 15;
                    float t[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        // rows are taken two at a time; the fence keeps the compiler from
                        // fetching all 120 coefficients up front (register pressure)
                        if ((i & 1) == 0) asm volatile("" ::: "memory");
                        float sacc = (i == c) ? 1.0f : 0.0f;
#pragma unroll
                        for (int j = 0; j < i; ++j) sacc = fmaf(-Ns[(o + i) * NP + o + j], t[j], sacc);
                        t[i] = sacc;
                    }
#pragma unroll
                    for (int i = 0; i < 16; ++i) Ns[(o + i) * NP + o + c] = t[i];
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                {
                    // T_21 = -T_22 (N_21 T_11); contraction length 16, upper k slots zero
                    bf16x8 a = zero8(), b = zero8();
                    if (g < 2) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            a[e] = (bf16)Ns[(16 + r16) * NP + 8 * g + e];
                            b[e] = (bf16)Ns[(8 * g + e) * NP + r16];
                        }
                    }
                    f32x4 tmp = {0.f, 0.f, 0.f, 0.f};
                    tmp = mfma16(a, b, tmp);
                    bf16x8 a2 = zero8(), b2 = zero8();
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        a2[e] = (bf16)Ns[(16 + r16) * NP + 16 + 4 * g + e];
                        b2[e] = (bf16)tmp[e];
                    }
                    f32x4 t21 = {0.f, 0.f, 0.f, 0.f};
                    t21 = mfma16(a2, b2, t21);
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) Ns[(16 + 4 * g + jj) * NP + r16] = -t21[jj];
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                {
                    const int row = lane >> 1, half = lane & 1;
                    bf16x8 lo, hi;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        lo[e] = (bf16)Ns[row * NP + 16 * half + e];
                        hi[e] = (bf16)Ns[row * NP + 16 * half + 8 + e];
                    }
                    st8(&Ts[(db * 32 + row) * TP + 16 * half], lo);
                    st8(&Ts[(db * 32 + row) * TP + 16 * half + 8], hi);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
        }
        __syncthreads();   // T blocks visible to everyone; scratch region free for the next phase

        // ------------------------------------------------------------ block forward substitution
        bf16x8 X[NB][NT];                      // finished blocks of this wave's slice, B-operand form

        // -G_ij for every j < i, transposed product so that lanes hold 4 consecutive j.
        auto gram_row = [&](int i, int buf) {
            bf16 *Gb = Gs + buf * 32 * GP;
            const int nh = w & 1;
            bf16x8 bk[NKS];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) bk[ks] = ld8(&Ks[(32 * i + 16 * nh + r16) * KP + 32 * ks + 8 * g]);
            const float nbeta = -bs[32 * i + 16 * nh + r16];
            for (int jt = (w >> 1); jt < 2 * i; jt += 8) {
                const bool two = jt + 4 < 2 * i;       // second tile of the pair exists
                const int jt2 = two ? jt + 4 : jt;
                f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    acc0 = mfma16(ld8(&Ks[(16 * jt + r16) * KP + 32 * ks + 8 * g]), bk[ks], acc0);
                    acc1 = mfma16(ld8(&Ks[(16 * jt2 + r16) * KP + 32 * ks + 8 * g]), bk[ks], acc1);
                }
                st4(&Gb[(16 * nh + r16) * GP + 16 * jt + 4 * g], cvt4(acc0 * nbeta));
                if (two) st4(&Gb[(16 * nh + r16) * GP + 16 * jt2 + 4 * g], cvt4(acc1 * nbeta));
            }
        };
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int buf = i & 1;
            if (i + 1 < NB) {
                gram_row(i + 1, buf ^ 1);
                stage_v(i + 1);
            }

            const bf16 *src = isV ? (Vs + buf * 32 * KP) : (Ks + 32 * i * KP);
            const bf16 *Gb = Gs + buf * 32 * GP;
            f32x4 acc[2][NT];
            // right-hand side beta_i (.) [K_i | V_i], read transposed into accumulator layout
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                f32x4 bt;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) bt[jj] = bs[32 * i + 16 * mi + 4 * g + jj];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    bf16x4 v = lds_read_tr4(&src[(16 * mi + 4 * g + (r16 >> 2)) * KP + cb + 16 * nt + 4 * (r16 & 3)]);
                    acc[mi][nt] = __builtin_convertvector(v, f32x4) * bt;
                }
            }
            // minus sum_j G_ij X_j  (G stored negated)
#pragma unroll
            for (int j = 0; j < i; ++j) {
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
                    bf16x8 a = join(ld4(&Gb[(16 * mi + r16) * GP + 32 * j + 4 * g]),
                                    ld4(&Gb[(16 * mi + r16) * GP + 32 * j + 16 + 4 * g]));
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) acc[mi][nt] = mfma16(a, X[j][nt], acc[mi][nt]);
                }
            }
            // X_i = T_ii R_i
            f32x4 xacc[2][NT];
            {
                bf16x8 rb[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) rb[nt] = join(cvt4(acc[0][nt]), cvt4(acc[1][nt]));
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
                    bf16x8 a = join(ld4(&Ts[(i * 32 + 16 * mi + r16) * TP + 4 * g]),
                                    ld4(&Ts[(i * 32 + 16 * mi + r16) * TP + 16 + 4 * g]));
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        f32x4 z = {0.f, 0.f, 0.f, 0.f};
                        xacc[mi][nt] = mfma16(a, rb[nt], z);
                    }
                }
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) X[i][nt] = join(cvt4(xacc[0][nt]), cvt4(xacc[1][nt]));

            if (isV) {
                // U' tiles are accumulator tiles as they stand: one contiguous 512 B store each
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        st4(Ug + ((size_t)((2 * i + mi) * DT + cb / 16 + nt) * 64 + lane) * 4, cvt4(xacc[mi][nt]));
            } else {
                // -W as A-operand tiles: transpose the 32 x FW tile through a wave-private LDS tile
                bf16 *Ws = WsAll + w * 32 * WP;
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        bf16x4 v = cvt4(-xacc[mi][nt]);
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) Ws[(16 * mi + 4 * g + jj) * WP + 16 * nt + r16] = v[jj];
                    }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                // this wave's columns are features [cb, cb + FW); lane (r16, g) of k-step ks holds
                // features 32 ks + 8 g .. + 7
                const int ks = cb / 32, fo = cb % 32;
                if (8 * g >= fo && 8 * g < fo + FW) {
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi)
                        st8(Wg + ((size_t)((2 * i + mi) * NKS + ks) * 64 + lane) * 8,
                            ld8(&Ws[(16 * mi + r16) * WP + 8 * g - fo]));
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
            __syncthreads();
        }

        // ------------------------------------------------------------ P = Mbar (.) Q K^T, Q tiles
#pragma unroll
        for (int q = 0; q < QV; ++q) {
            const int v = tid + NTHR * q;
            if ((q + 1) * NTHR <= C * D / 8 || v < C * D / 8) st8(&Qs[(v / VPR) * KP + (v % VPR) * 8], qreg[q]);
        }
        __syncthreads();
        if (more) fetch_q(nxt);
        for (int it = w; it < CT * NKT; it += kFlowWaves) {
            const int tt = it / NKT, kt = it % NKT;
            if (32 * kt >= R * (16 * tt + 16)) continue;       // wholly after the last visible token
            bf16x8 bq[NKS];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) bq[ks] = ld8(&Qs[(16 * tt + r16) * KP + 32 * ks + 8 * g]);
            if (kt == 0) {
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) st8(Qtg + ((size_t)(tt * NKS + ks) * 64 + lane) * 8, bq[ks]);
            }
            f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                acc0 = mfma16(ld8(&Ks[(32 * kt + r16) * KP + 32 * ks + 8 * g]), bq[ks], acc0);
                acc1 = mfma16(ld8(&Ks[(32 * kt + 16 + r16) * KP + 32 * ks + 8 * g]), bq[ks], acc1);
            }
            const int t = 16 * tt + r16;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                if ((32 * kt + 4 * g + jj) / R > t) acc0[jj] = 0.0f;
                if ((32 * kt + 16 + 4 * g + jj) / R > t) acc1[jj] = 0.0f;
            }
            st8(Ptg + ((size_t)(tt * NKT + kt) * 64 + lane) * 8, join(cvt4(acc0), cvt4(acc1)));
        }
        __syncthreads();   // every read of this chunk's K, Q is done before the next chunk lands
    }
}

// ---------------------------------------------------------------------------- host side
#define PF_FLOW_INSTANCES(X) \
    X(64, 64, 64) X(64, 128, 64) X(64, 128, 128) X(64, 256, 64) X(64, 256, 128) \
    X(128, 64, 64) X(128, 128, 64) X(128, 128, 128) X(128, 256, 64) X(128, 256, 128)

bool mfma_instance_exists(int d, int n, int chunk)
{
#define X(DD, NN, CC) if (d == DD && n == NN && chunk == CC) return true;
    PF_FLOW_INSTANCES(X)
#undef X
    return false;
}

template <int D, int N, int C>
static hipError_t launch_flow_instance(const void *Q, const void *K, const void *V, const void *beta,
                                       void *Wt, void *Ut, void *Kt, void *Pt, void *Qt, size_t nchunks,
                                       hipStream_t stream)
{
    auto kern = flow_kernel<D, N, C>;
    constexpr size_t lds = FlowLds<D, N, C>::total;
    static_assert(lds <= kMaxLdsBytes, "flow kernel LDS plan exceeds the CU");
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    // Persistent grid: as many workgroups as the chip holds at once (LDS decides how many per
    // CU), each walking its share of the chunks.
    const size_t per_cu = kMaxLdsBytes / lds ? kMaxLdsBytes / lds : 1;
    const size_t resident = kNumCUs * (per_cu > 2 ? 2 : per_cu);
    const unsigned grid = (unsigned)(nchunks < resident ? nchunks : resident);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kFlowThreads), lds, stream, (const bf16 *)Q,
                       (const bf16 *)K, (const bf16 *)V, (const bf16 *)beta, (bf16 *)Wt, (bf16 *)Ut,
                       (bf16 *)Kt, (bf16 *)Pt, (bf16 *)Qt, (int)nchunks);
    return hipGetLastError();
}

hipError_t launch_chunk_flow(const void *Q, const void *K, const void *V, const void *beta, void *Wt,
                             void *Ut, void *Kt, void *Pt, void *Qt, int heads, int L, int d, int r,
                             int chunk, hipStream_t stream)
{
    const size_t nchunks = (size_t)heads * (L / chunk);
    if (nchunks == 0) return hipSuccess;
    if (nchunks > 0x7fffffffull) return hipErrorInvalidValue;
    const int n = chunk * r;
#define X(DD, NN, CC)                                                                                 \
    if (d == DD && n == NN && chunk == CC)                                                             \
        return launch_flow_instance<DD, NN, CC>(Q, K, V, beta, Wt, Ut, Kt, Pt, Qt, nchunks, stream);
    PF_FLOW_INSTANCES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace pf
