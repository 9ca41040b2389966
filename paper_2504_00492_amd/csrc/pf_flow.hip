// Chunk-flow kernel: step 2 of Section 3 of ParallelFlow (arXiv 2504.00492), "parallel
// compute".  Persistent workgroups (8 wavefronts) walk the (b, h, chunk) triples; chunks do not
// depend on each other.
//
// In delta variables (Remark in Section 3.1: A = beta k, Atil = -beta v, B = -k) Theorem 3.2
// reads, with n = chunk * r virtual tokens and M strict in time,
//     W = T (beta (.) K),   U' = T (beta (.) V),   T = (Id + G)^{-1},   G = M (.) diag(beta) K K^T,
// where U' = -U.  What the state hand-over needs of the chunk is U' - W S^T = T (beta (.) (V - K S^T)),
// so T itself is the compact form that is handed on: n x n lower block-triangular, which is
// smaller than W and U' together, and it depends on K and beta only.
//
// T is obtained by the block substitution of Proposition 3.3 on 32-row blocks, run on the
// transposed system  (Id + G)^T X = Id  (X = T^T, upper block-triangular, solved from the last
// block up):
//     X_j = T_jj^T ( E_j  -  sum_{i > j} G_ij^T X_i ).
// Solving for T^T rather than T is a layout choice: an MFMA accumulator tile of X (4 consecutive
// rows of T^T per lane) is 4 consecutive columns of one row of T, which is the A-operand form
// the scan kernel wants, so finished tiles go from registers straight to their place in the
// hand-over array.  T_jj (32 x 32) comes from two 16 x 16 forward substitutions in fp32 on the
// vector ALU and one block merge T_21 = -T_22 G_21 T_11 on MFMA.
//
// Work split.  The n columns of X (= rows of T) are dealt to the waves in 16-column slices; a
// wave keeps the finished blocks X_i of its slices in registers, already in B-operand form (see
// pf_common.h), so the substitution needs no LDS traffic for X.  G^T block-columns and T_jj^T
// are built cooperatively and read by all waves as A operands from LDS.  P = Mbar (.) Q K^T
// (readout mask, inclusive in time) is computed from the same resident K.
//
// While a chunk is processed, K, beta and Q of the workgroup's next chunk are already on their
// way from HBM into registers.
//
// Outputs: the tiled operand arrays Tt and Pt described in pf_layout.h.
#include "pf_internal.h"
#include "pf_common.h"
#include "pf_layout.h"

#include <atomic>

namespace pf {

constexpr int kFlowThreads = 512;
constexpr int kFlowWaves = kFlowThreads / 64;

// GEN: general drivers (A, Atil, B) of Section 3.1 instead of the delta mapping: the rows of the
// system matrix come from A and its columns from B, so two n x d arrays are resident instead of K.
template <int D, int N, int C, bool GEN = false>
struct FlowLds {
    static constexpr int NB = N / 32;       // 32-row blocks per chunk
    static constexpr int KP = D + 8;        // pitch of K / Q rows (bf16)
    static constexpr int GP = N + 8;        // pitch of a row of a G^T block-column (bf16)
    static constexpr int TP = 40;           // pitch of a T_jj^T row (bf16)
    static constexpr int NP = 36;           // pitch of the fp32 scratch used to build T_jj
    static constexpr size_t oKs = 0;                                    // K; with GEN: B, then A
    static constexpr size_t oBs = oKs + (size_t)(GEN ? 2 : 1) * N * KP * 2;
    static constexpr size_t oTs = oBs + (size_t)N * 4;
    static constexpr size_t oUn = oTs + (size_t)NB * 32 * TP * 2;       // region reused by phase
    // phase "build T_jj": fp32 scratch, one 32 x NP tile per wave that has a diagonal block
    static constexpr size_t szNs = (size_t)(NB < kFlowWaves ? NB : kFlowWaves) * 32 * NP * 4;
    // phase "substitute": G^T block-column (x2)
    static constexpr size_t szG = (size_t)2 * 32 * GP * 2;
    // phase "P": the chunk's queries
    static constexpr size_t szQ = (size_t)C * KP * 2;
    static constexpr size_t szUn = szNs > szG ? (szNs > szQ ? szNs : szQ) : (szG > szQ ? szG : szQ);
    static constexpr size_t total = oUn + szUn;
};

template <int D, int N, int C, bool GEN = false>
__global__ __launch_bounds__(kFlowThreads) void flow_kernel(
    const bf16 *__restrict__ Q, const bf16 *__restrict__ K, const bf16 *__restrict__ beta,
    bf16 *__restrict__ Tt, bf16 *__restrict__ Pt, int nchunks, int NC, int tail, int mask_shift)
{
    // With GEN, K is the array of B rows and `beta` the array of A rows (n x d, like K); the
    // system matrix is Id - M (.) A B^T and P = Mbar (.) Q B^T (Theorem 3.2 as printed).
    using Ld = FlowLds<D, N, C, GEN>;
    constexpr int R = N / C;          // rank: virtual tokens per token
    constexpr int NB = Ld::NB;
    constexpr int NKS = D / 32, NKT = N / 32, CT = C / 16;
    constexpr int KP = Ld::KP, GP = Ld::GP, TP = Ld::TP, NP = Ld::NP;
    constexpr int NTHR = kFlowThreads;
    constexpr int NS = N / 16;                                          // 16-column slices of X
    constexpr int SPW = (NS + kFlowWaves - 1) / kFlowWaves;             // slices per wave
    static_assert(32 % R == 0 && N % 32 == 0 && C % 16 == 0 && D % 32 == 0, "tile shapes");
    static_assert(SPW <= 2, "a wave owns at most two slices");

    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16 *Ks = reinterpret_cast<bf16 *>(smem + Ld::oKs);             // column side of the Gram: K, or B
    bf16 *As = GEN ? Ks + N * KP : Ks;                               // row side: K, or A
    float *bs = reinterpret_cast<float *>(smem + Ld::oBs);
    bf16 *Ts = reinterpret_cast<bf16 *>(smem + Ld::oTs);
    float *NsAll = reinterpret_cast<float *>(smem + Ld::oUn);
    bf16 *Gs = reinterpret_cast<bf16 *>(smem + Ld::oUn);
    bf16 *Qs = reinterpret_cast<bf16 *>(smem + Ld::oUn);

    const int tid0 = threadIdx.x;

    // ---- register sets that carry the next chunk's inputs
    constexpr int VPR = D / 8;                         // 16-byte vectors per row
    constexpr int KV = (N * D / 8 + NTHR - 1) / NTHR;  // vectors of K per thread
    constexpr int QV = (C * D / 8 + NTHR - 1) / NTHR;  // vectors of Q per thread
    bf16x8 kreg[KV], qreg[QV], areg[GEN ? KV : 1];
    bf16 breg = (bf16)0.0f;   // kept as loaded: converting here would wait for the fetch
    static_assert(N <= NTHR, "beta of a chunk is fetched by one pass");

    // A head holds NC whole blocks followed by `tail` tokens that another kernel takes: block c
    // of the compact numbering starts (c / NC) * tail tokens further on in Q, K, beta.
    auto skew = [&](size_t c) { return tail ? (c / (size_t)NC) * (size_t)tail : (size_t)0; };
    auto fetch_k = [&](size_t c) {
        const bf16 *Kg = K + (c * (size_t)N + skew(c) * R) * D;
#pragma unroll
        for (int q = 0; q < KV; ++q) {
            const int v = tid0 + NTHR * q;
            if ((q + 1) * NTHR <= N * D / 8 || v < N * D / 8) {
                kreg[q] = ld8(Kg + (size_t)v * 8);
                if constexpr (GEN) areg[q] = ld8(beta + (c * (size_t)N + skew(c) * R) * D + (size_t)v * 8);
            }
        }
        if constexpr (!GEN)
            breg = beta[c * (size_t)N + skew(c) * R + (tid0 % N)];   // every thread loads: no branch, always in range
    };
    auto fetch_q = [&](size_t c) {
        const bf16 *Qg = Q + (c * (size_t)C + skew(c)) * D;
#pragma unroll
        for (int q = 0; q < QV; ++q) {
            const int v = tid0 + NTHR * q;
            if ((q + 1) * NTHR <= C * D / 8 || v < C * D / 8) qreg[q] = ld8(Qg + (size_t)v * 8);
        }
    };

    size_t cid = blockIdx.x;
    if (cid < (size_t)nchunks) {
        fetch_k(cid);
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
        // The fetch for "the next chunk" is unconditional (the last chunk re-fetches itself): a
        // branch around a load makes every later wait assume the shorter queue.
        const size_t nxt = cid + gridDim.x < (size_t)nchunks ? cid + gridDim.x : cid;
        bf16 *Ttg = Tt + cid * (size_t)N * N;
        bf16 *Ptg = Pt + cid * (size_t)C * N;

        // ------------------------------------------------------------ K, beta: registers -> LDS
#pragma unroll
        for (int q = 0; q < KV; ++q) {
            const int v = tid + NTHR * q;
            if ((q + 1) * NTHR <= N * D / 8 || v < N * D / 8) {
                st8(&Ks[(v / VPR) * KP + (v % VPR) * 8], kreg[q]);
                if constexpr (GEN) st8(&As[(v / VPR) * KP + (v % VPR) * 8], areg[q]);
            }
        }
        // the row factor of the system matrix: beta_i for the delta rule (G_ij = beta_i k_i . k_j);
        // -1 for general drivers (G_ij = -a_i . b_j)
        if (tid < N) bs[tid] = GEN ? -1.0f : (float)breg;
        __syncthreads();
        fetch_k(nxt);

        // ------------------------------------------------------------ T_jj^T for every 32-block
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
                    bf16x8 a0 = k0, a1 = k1;
                    if constexpr (GEN) {
                        a0 = ld8(&As[(32 * db + r16) * KP + 32 * ks + 8 * g]);
                        a1 = ld8(&As[(32 * db + 16 + r16) * KP + 32 * ks + 8 * g]);
                    }
                    acc[0] = mfma16(a0, k0, acc[0]);   // rows 0-15,  cols 0-15
                    acc[1] = mfma16(a1, k0, acc[1]);   // rows 16-31, cols 0-15
                    acc[2] = mfma16(a1, k1, acc[2]);   // rows 16-31, cols 16-31
                }
#pragma unroll
                for (int tile = 0; tile < 4; ++tile) {
                    const int mi = tile >> 1, ni = tile & 1;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const int row = 16 * mi + 4 * g + jj, col = 16 * ni + r16;
                        float val = 0.0f;
                        // strict in time: rows and columns compared by token, i.e. by virtual
                        // token >> log2(R); mask_shift = 0 compares virtual tokens themselves
                        // (the r sub-updates of a token then see each other, one after another)
                        if (tile != 1 && ((col >> mask_shift) < (row >> mask_shift)))
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
                    // store the block transposed: row of the stored tile = column of T_jj
                    const int row = lane >> 1, half = lane & 1;
                    bf16x8 lo, hi;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        lo[e] = (bf16)Ns[(16 * half + e) * NP + row];
                        hi[e] = (bf16)Ns[(16 * half + 8 + e) * NP + row];
                    }
                    st8(&Ts[(db * 32 + row) * TP + 16 * half], lo);
                    st8(&Ts[(db * 32 + row) * TP + 16 * half + 8], hi);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
        }
        __syncthreads();   // T blocks visible to everyone; scratch region free for the next phase

        // ------------------------------------------------------------ block substitution, last block first
        // Slice ownership: wave w has slice w and (when there are 16 slices) slice 15 - w, which
        // evens out the triangular amount of work.
        bf16x8 X[SPW][NB];   // finished blocks of this wave's slices, B-operand form

        // -G^T block-column j: rows b = the 32 tokens of block j, columns a = every later token.
        // Product taken as (rows a) x (cols b) so that lanes hold 4 consecutive a.
        auto gram_col = [&](int j, int buf) {
            bf16 *Gb = Gs + buf * 32 * GP;
            const int nh = w & 1;
            bf16x8 bk[NKS];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) bk[ks] = ld8(&Ks[(32 * j + 16 * nh + r16) * KP + 32 * ks + 8 * g]);
            for (int at = 2 * (j + 1) + (w >> 1); at < 2 * NB; at += 8) {
                const bool two = at + 4 < 2 * NB;       // second tile of the pair exists
                const int at2 = two ? at + 4 : at;
                f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    acc0 = mfma16(ld8(&As[(16 * at + r16) * KP + 32 * ks + 8 * g]), bk[ks], acc0);
                    acc1 = mfma16(ld8(&As[(16 * at2 + r16) * KP + 32 * ks + 8 * g]), bk[ks], acc1);
                }
                f32x4 nb0, nb1;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    nb0[e] = -bs[16 * at + 4 * g + e];
                    nb1[e] = -bs[16 * at2 + 4 * g + e];
                }
                st4(&Gb[(16 * nh + r16) * GP + 16 * at + 4 * g], cvt4(acc0 * nb0));
                if (two) st4(&Gb[(16 * nh + r16) * GP + 16 * at2 + 4 * g], cvt4(acc1 * nb1));
            }
        };

        // Block j reads column j of G^T from buffer j & 1.  The last block has no later block and
        // needs none; column NB - 2 is built here, and every later step builds the column of the
        // step after it into the other buffer.
        if (NB > 1) gram_col(NB - 2, (NB - 2) & 1);
        __syncthreads();
#pragma unroll
        for (int step = 0; step < NB; ++step) {
            const int j = NB - 1 - step;
            const int buf = j & 1;
            if (step > 0 && j > 0) gram_col(j - 1, (j - 1) & 1);
            const bf16 *Gb = Gs + buf * 32 * GP;
#pragma unroll
            for (int sl = 0; sl < SPW; ++sl) {
                const int s = sl == 0 ? w : NS - 1 - w;          // slice: columns 16 s .. 16 s + 15 of X
                const bool have = sl == 0 ? (w < NS) : true;
                const int ib = s >> 1;                            // block that holds the slice's diagonal
                if (have && ib >= j) {                            // otherwise X_j is zero on this slice
                    f32x4 acc[2];
                    // right-hand side E_j: the identity, non-zero only on the slice's own block
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            acc[mi][e] = (ib == j && (s & 1) == mi && 4 * g + e == r16) ? 1.0f : 0.0f;
                    // minus sum_{i > j} G_ij^T X_i  (G stored negated); X_i = 0 beyond the slice's block
#pragma unroll
                    for (int i = 0; i < NB; ++i) {
                        if (i > j && i <= ib) {
#pragma unroll
                            for (int mi = 0; mi < 2; ++mi) {
                                bf16x8 a = join(ld4(&Gb[(16 * mi + r16) * GP + 32 * i + 4 * g]),
                                                ld4(&Gb[(16 * mi + r16) * GP + 32 * i + 16 + 4 * g]));
                                acc[mi] = mfma16(a, X[sl][i], acc[mi]);
                            }
                        }
                    }
                    // X_j = T_jj^T R_j
                    bf16x8 rb = join(cvt4(acc[0]), cvt4(acc[1]));
                    f32x4 xacc[2];
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi) {
                        bf16x8 a = join(ld4(&Ts[(j * 32 + 16 * mi + r16) * TP + 4 * g]),
                                        ld4(&Ts[(j * 32 + 16 * mi + r16) * TP + 16 + 4 * g]));
                        f32x4 z = {0.f, 0.f, 0.f, 0.f};
                        xacc[mi] = mfma16(a, rb, z);
                    }
                    X[sl][j] = join(cvt4(xacc[0]), cvt4(xacc[1]));
                    // lane (r16, g) now holds T[16 s + r16][32 j + 4 g + e] (e < 4) and
                    // T[16 s + r16][32 j + 16 + 4 g + e - 4] (e >= 4): the A-operand tile (s, j) as is.
                    st8(Ttg + full_tile_offset(NKT, s, j) + lane * 8, X[sl][j]);
                }
            }
            __syncthreads();
        }

        // ------------------------------------------------------------ P = Mbar (.) Q K^T
#pragma unroll
        for (int q = 0; q < QV; ++q) {
            const int v = tid + NTHR * q;
            if ((q + 1) * NTHR <= C * D / 8 || v < C * D / 8) st8(&Qs[(v / VPR) * KP + (v % VPR) * 8], qreg[q]);
        }
        __syncthreads();
        fetch_q(nxt);
        for (int it = w; it < CT * NKT; it += kFlowWaves) {
            const int tt = it / NKT, kt = it % NKT;
            if (32 * kt >= R * (16 * tt + 16)) continue;       // wholly after the last visible token
            bf16x8 bq[NKS];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) bq[ks] = ld8(&Qs[(16 * tt + r16) * KP + 32 * ks + 8 * g]);
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
            st8(Ptg + full_tile_offset(NKT, tt, kt) + lane * 8, join(cvt4(acc0), cvt4(acc1)));
        }
        __syncthreads();   // every read of this chunk's K, Q is done before the next chunk lands
    }
}

// ---------------------------------------------------------------------------- host side
#define PF_FLOW_INSTANCES(X) \
    X(64, 64, 64) X(64, 64, 32) X(64, 128, 32) X(64, 128, 64) X(64, 128, 128) X(64, 256, 64) X(64, 256, 128) \
    X(128, 64, 64) X(128, 64, 32) X(128, 128, 32) X(128, 128, 64) X(128, 128, 128) X(128, 256, 64) X(128, 256, 128)

bool mfma_instance_exists(int d, int n, int chunk)
{
#define X(DD, NN, CC) if (d == DD && n == NN && chunk == CC) return true;
    PF_FLOW_INSTANCES(X)
#undef X
    return false;
}

template <int D, int N, int C, bool GEN = false>
static hipError_t launch_flow_instance(const void *Q, const void *K, const void *beta, void *Tt, void *Pt,
                                       size_t nchunks, int NC, int tail, bool product, hipStream_t stream)
{
    auto kern = flow_kernel<D, N, C, GEN>;
    int mask_shift = 0;
    if (!product)
        while ((1 << mask_shift) < N / C) ++mask_shift;
    constexpr size_t lds = FlowLds<D, N, C, GEN>::total;
    static_assert(lds <= kMaxLdsBytes, "flow kernel LDS plan exceeds the CU");
    static std::atomic<uint64_t> armed{0};
    hipError_t e = arm_dynamic_lds(armed, reinterpret_cast<const void *>(kern), lds);
    if (e != hipSuccess) return e;
    // Persistent grid: as many workgroups as the chip holds at once (LDS decides how many per
    // CU, at most two), each walking its share of the chunks.
    const size_t per_cu = kMaxLdsBytes / lds ? kMaxLdsBytes / lds : 1;
    const size_t resident = (size_t)device_cu_count() * (per_cu > 2 ? 2 : per_cu);
    const unsigned grid = (unsigned)(nchunks < resident ? nchunks : resident);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kFlowThreads), lds, stream, (const bf16 *)Q,
                       (const bf16 *)K, (const bf16 *)beta, (bf16 *)Tt, (bf16 *)Pt, (int)nchunks, NC, tail, mask_shift);
    return hipGetLastError();
}

hipError_t launch_chunk_flow(const void *Q, const void *K, const void *beta, void *Tt, void *Pt,
                             int heads, int L, int d, int r, int chunk, hipStream_t stream, bool product)
{
    const int NC = L / chunk, tail = L % chunk;   // the tail tokens of every head are skipped
    const size_t nchunks = (size_t)heads * NC;
    if (nchunks == 0) return hipSuccess;
    if (nchunks > 0x7fffffffull) return hipErrorInvalidValue;
    const int n = chunk * r;
#define X(DD, NN, CC)                                                                        \
    if (d == DD && n == NN && chunk == CC)                                                    \
        return launch_flow_instance<DD, NN, CC>(Q, K, beta, Tt, Pt, nchunks, NC, tail, product, stream);
    PF_FLOW_INSTANCES(X)
#undef X
    return hipErrorInvalidValue;
}

bool mfma_general_instance_exists(int d, int n, int chunk) { return n <= 128 && mfma_instance_exists(d, n, chunk); }

hipError_t launch_chunk_flow_general(const void *Q, const void *A, const void *Bm, void *Tt, void *Pt, int heads,
                                     int L, int d, int r, int chunk, hipStream_t stream)
{
    const int NC = L / chunk, tail = L % chunk;   // the tail tokens of every head are skipped
    const size_t nchunks = (size_t)heads * NC;
    if (nchunks == 0) return hipSuccess;
    if (nchunks > 0x7fffffffull) return hipErrorInvalidValue;
    const int n = chunk * r;
#define X(DD, NN, CC)                                                                                    \
    if constexpr (NN <= 128) {                                                                            \
        if (d == DD && n == NN && chunk == CC)                                                            \
            return launch_flow_instance<DD, NN, CC, true>(Q, Bm, A, Tt, Pt, nchunks, NC, tail, false, stream); \
    }
    PF_FLOW_INSTANCES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace pf
