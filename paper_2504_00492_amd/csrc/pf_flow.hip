// Chunk-flow kernel: step 2 of Section 3 of ParallelFlow (arXiv 2504.00492), "parallel
// compute".  One workgroup (4 wavefronts) per (b, h, chunk); no dependence between chunks.
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
// Work split.  The 2 d right-hand-side columns are dealt to the 4 wavefronts (waves 0-1 the
// key columns, waves 2-3 the value columns).  A wave keeps every finished X_j of its column
// slice in registers, already in MFMA B-operand form, so the substitution itself needs no
// barrier and no LDS traffic for X.  G_ij and T_ii are built cooperatively and read by all
// waves as A operands from LDS.  Gram blocks are computed transposed so that an accumulator
// tile (4 consecutive j per lane) goes to row-major LDS with 8-byte writes.
//
// Outputs (bf16):  Wneg = -W  row-major [n][d];  UpT = U'^T [d][n];  KT = K^T [d][n];
//                  P = Mbar (.) Q K^T  [chunk][n], Mbar inclusive in time (readout mask).
#include "pf_internal.h"
#include "pf_common.cuh"

namespace pf {

template <int D, int N>
struct FlowLds {
    static constexpr int NB = N / 32;       // 32-row blocks per chunk
    static constexpr int KP = D + 8;        // pitch of K / V rows (bf16)
    static constexpr int GP = N + 8;        // pitch of a G block-row (bf16)
    static constexpr int TP = 40;           // pitch of a T_ii row (bf16)
    static constexpr int NP = 36;           // pitch of the fp32 scratch used to build T_ii
    static constexpr int WP = D / 2 + 8;    // pitch of the per-wave W staging tile (bf16)
    static constexpr size_t oKs = 0;
    static constexpr size_t oBs = oKs + (size_t)N * KP * 2;
    static constexpr size_t oTs = oBs + (size_t)N * 4;
    static constexpr size_t oUn = oTs + (size_t)NB * 32 * TP * 2;       // union region
    // union, phase "build T": fp32 scratch, one 32 x NP tile per wave
    static constexpr size_t szNs = (size_t)4 * 32 * NP * 4;
    // union, phase "substitute": V block (x2), G block-row (x2), W staging (2 waves)
    static constexpr size_t oVs = oUn;
    static constexpr size_t oGs = oVs + (size_t)2 * 32 * KP * 2;
    static constexpr size_t oWs = oGs + (size_t)2 * 32 * GP * 2;
    static constexpr size_t endS = oWs + (size_t)2 * 32 * WP * 2;
    static constexpr size_t total = (endS > oUn + szNs) ? endS : oUn + szNs;
};

template <int D, int N, int C>
__global__ __launch_bounds__(256) void flow_kernel(const bf16 *__restrict__ Q, const bf16 *__restrict__ K,
                                                   const bf16 *__restrict__ V, const bf16 *__restrict__ beta,
                                                   bf16 *__restrict__ Wneg, bf16 *__restrict__ UpT,
                                                   bf16 *__restrict__ KT, bf16 *__restrict__ P)
{
    using Ld = FlowLds<D, N>;
    constexpr int R = N / C;          // rank: virtual tokens per token
    constexpr int NB = Ld::NB;
    constexpr int NT = D / 32;        // 16-column tiles of the right-hand side per wave
    constexpr int NKS = D / 32;       // k-steps of a contraction over d
    constexpr int KP = Ld::KP, GP = Ld::GP, TP = Ld::TP, NP = Ld::NP, WP = Ld::WP;
    static_assert(32 % R == 0 && N % 32 == 0 && C % 16 == 0 && D % 32 == 0, "tile shapes");

    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16 *Ks = reinterpret_cast<bf16 *>(smem + Ld::oKs);
    float *bs = reinterpret_cast<float *>(smem + Ld::oBs);
    bf16 *Ts = reinterpret_cast<bf16 *>(smem + Ld::oTs);
    float *NsAll = reinterpret_cast<float *>(smem + Ld::oUn);
    bf16 *Vs = reinterpret_cast<bf16 *>(smem + Ld::oVs);
    bf16 *Gs = reinterpret_cast<bf16 *>(smem + Ld::oGs);
    bf16 *WsAll = reinterpret_cast<bf16 *>(smem + Ld::oWs);

    const int tid = threadIdx.x;
    const int w = tid >> 6, lane = tid & 63;
    const int r16 = lane & 15, g = lane >> 4;

    const size_t cid = blockIdx.x;
    const bf16 *Kg = K + cid * (size_t)N * D;
    const bf16 *Vg = V + cid * (size_t)N * D;
    const bf16 *bg = beta + cid * (size_t)N;
    const bf16 *Qg = Q + cid * (size_t)C * D;
    bf16 *Wg = Wneg + cid * (size_t)N * D;
    bf16 *Ug = UpT + cid * (size_t)N * D;
    bf16 *KTg = KT + cid * (size_t)N * D;
    bf16 *Pg = P + cid * (size_t)C * N;

    // ---------------------------------------------------------------- load K, beta
    for (int v = tid; v < N * D / 8; v += 256) {
        const int row = v / (D / 8), cg = v % (D / 8);
        st8(&Ks[row * KP + cg * 8], ld8(Kg + (size_t)row * D + cg * 8));
    }
    for (int i = tid; i < N; i += 256) bs[i] = (float)bg[i];
    __syncthreads();

    // ---------------------------------------------------------------- K^T out
    for (int idx = tid; idx < D * (N / 8); idx += 256) {
        const int x = idx % D, tg = idx / D;
        bf16x8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = Ks[(8 * tg + e) * KP + x];
        st8(KTg + (size_t)x * N + 8 * tg, v);
    }

    // ---------------------------------------------------------------- T_ii for every 32-block
    {
        float *Ns = NsAll + w * 32 * NP;
        for (int it = 0; it < (NB + 3) / 4; ++it) {
            const int db = it * 4 + w;
            const bool active = db < NB;
            if (active) {
                // N_db = strict-in-time part of diag(beta) K K^T on the block, fp32, row-major
#pragma unroll
                for (int tile = 0; tile < 4; ++tile) {
                    const int mi = tile >> 1, ni = tile & 1;
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                    if (!(mi == 0 && ni == 1)) {
#pragma unroll
                        for (int ks = 0; ks < NKS; ++ks) {
                            bf16x8 a = ld8(&Ks[(32 * db + 16 * mi + r16) * KP + 32 * ks + 8 * g]);
                            bf16x8 b = ld8(&Ks[(32 * db + 16 * ni + r16) * KP + 32 * ks + 8 * g]);
                            acc = mfma16(a, b, acc);
                        }
                    }
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        const int row = 16 * mi + 4 * g + jj, col = 16 * ni + r16;
                        const float val = (col / R < row / R) ? acc[jj] * bs[32 * db + row] : 0.0f;
                        Ns[row * NP + col] = val;
                    }
                }
            }
            __syncthreads();
            if (active && lane < 32) {
                // two 16 x 16 unit-lower-triangular inverses, lane = (sub-block, column)
                const int o = 16 * (lane >> 4), c = lane & 15;
                float t[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float s = (i == c) ? 1.0f : 0.0f;
#pragma unroll
                    for (int j = 0; j < i; ++j) s = fmaf(-Ns[(o + i) * NP + o + j], t[j], s);
                    t[i] = s;
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) Ns[(o + i) * NP + o + c] = t[i];
            }
            __syncthreads();
            if (active) {
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
            __syncthreads();
            if (active) {
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
            __syncthreads();
        }
    }

    // ---------------------------------------------------------------- block forward substitution
    const bool isV = (w >> 1) != 0;        // waves 2,3 solve for U', waves 0,1 for W
    const int cb = (w & 1) * (D / 2);      // first column of this wave's slice inside K or V
    bf16x8 X[NB][NT];                      // finished blocks of this wave's slice, B-operand form

    auto produce = [&](int i, int buf) {
        // V rows of block i
        bf16 *Vb = Vs + buf * 32 * KP;
        for (int v = tid; v < 32 * D / 8; v += 256) {
            const int row = v / (D / 8), cg = v % (D / 8);
            st8(&Vb[row * KP + cg * 8], ld8(Vg + (size_t)(32 * i + row) * D + cg * 8));
        }
        // -G_ij for every j < i, transposed product so that lanes hold 4 consecutive j
        bf16 *Gb = Gs + buf * 32 * GP;
        const int nh = w & 1;
        bf16x8 bk[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) bk[ks] = ld8(&Ks[(32 * i + 16 * nh + r16) * KP + 32 * ks + 8 * g]);
        const float nbeta = -bs[32 * i + 16 * nh + r16];
        for (int jt = (w >> 1); jt < 2 * i; jt += 2) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                acc = mfma16(ld8(&Ks[(16 * jt + r16) * KP + 32 * ks + 8 * g]), bk[ks], acc);
            st4(&Gb[(16 * nh + r16) * GP + 16 * jt + 4 * g], cvt4(acc * nbeta));
        }
    };

    produce(0, 0);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int buf = i & 1;
        if (i + 1 < NB) produce(i + 1, buf ^ 1);

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
            // U'^T: 4 consecutive tokens of one feature = one 8-byte store
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    st4(Ug + (size_t)(cb + 16 * nt + r16) * N + 32 * i + 16 * mi + 4 * g, cvt4(xacc[mi][nt]));
        } else {
            // -W row-major: transpose the 32 x (d/2) tile through a wave-private LDS tile
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
            const int row = lane >> 1, half = lane & 1;
#pragma unroll
            for (int q = 0; q < D / 32; ++q)
                st8(Wg + (size_t)(32 * i + row) * D + cb + half * (D / 4) + 8 * q,
                    ld8(&Ws[row * WP + half * (D / 4) + 8 * q]));
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        __syncthreads();
    }

    // ---------------------------------------------------------------- P = Mbar (.) Q K^T
    for (int tt = w; tt < C / 16; tt += 4) {
        bf16x8 bq[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) bq[ks] = ld8(Qg + (size_t)(16 * tt + r16) * D + 32 * ks + 8 * g);
        const int t = 16 * tt + r16;
        for (int jt = 0; jt < N / 16; ++jt) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            if ((16 * jt) / R <= 16 * tt + 15) {
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks)
                    acc = mfma16(ld8(&Ks[(16 * jt + r16) * KP + 32 * ks + 8 * g]), bq[ks], acc);
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
                    if ((16 * jt + 4 * g + jj) / R > t) acc[jj] = 0.0f;
            }
            st4(Pg + (size_t)t * N + 16 * jt + 4 * g, cvt4(acc));
        }
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
                                       void *Wneg, void *UpT, void *KT, void *P, size_t nchunks,
                                       hipStream_t stream)
{
    auto kern = flow_kernel<D, N, C>;
    constexpr size_t lds = FlowLds<D, N>::total;
    static_assert(lds <= kMaxLdsBytes, "flow kernel LDS plan exceeds the CU");
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)nchunks), dim3(256), lds, stream, (const bf16 *)Q,
                       (const bf16 *)K, (const bf16 *)V, (const bf16 *)beta, (bf16 *)Wneg, (bf16 *)UpT,
                       (bf16 *)KT, (bf16 *)P);
    return hipGetLastError();
}

hipError_t launch_chunk_flow(const void *Q, const void *K, const void *V, const void *beta, void *Wneg,
                             void *UpT, void *KT, void *P, int heads, int L, int d, int r, int chunk,
                             hipStream_t stream)
{
    const size_t nchunks = (size_t)heads * (L / chunk);
    if (nchunks == 0) return hipSuccess;
    if (nchunks > 0x7fffffffull) return hipErrorInvalidValue;
    const int n = chunk * r;
#define X(DD, NN, CC)                                                                              \
    if (d == DD && n == NN && chunk == CC)                                                          \
        return launch_flow_instance<DD, NN, CC>(Q, K, V, beta, Wneg, UpT, KT, P, nchunks, stream);
    PF_FLOW_INSTANCES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace pf
