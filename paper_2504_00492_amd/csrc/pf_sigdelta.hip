// W and U of every chunk by the grid recursion of Theorem 3.4 (ParallelFlow, arXiv 2504.00492),
// swept along anti-diagonals, with no triangular inverse anywhere.  An alternative to the blocked
// substitution of pf_flow.hip for step 2 of Section 3; it exists to be measured against it.
//
// In delta variables (Remark in Section 3.1: A = beta k, Atil = -beta v, B = -k) and row form
// (a token's r columns are r rows of length d), with X = [A | Atil] (d_k + d_v columns) and
// Gm[(m, j'), (k, j)] = b_{m,j'} . a_{k,j} = -beta_{k,j} (k_{m,j'} . k_{k,j}), the grid values
// Y(m, k) (r rows each, 0 <= m <= k < C) obey
//
//   Y(0, k)     = X_k
//   Y(m, m)     = Y(m-1, m) + Gm[m-1, m]^T-weighted rows of Y(m-1, m-1)
//   Y(m, k)     = Y(m-1, k) + Y(m, k-1) - Y(m-1, k-1)
//                 + (Gm[m-1, k] - Gm[m-1, k-1])-weighted rows of Y(m-1, m-1)         (m < k)
//
// ("weighted rows": row j of the result gains sum_j' coef[j'][j] * row j' of the diagonal value),
// and the diagonal Y(k, k) is [W_k | U_k] of Theorem 3.2.  The same recursion serves W and U
// because both solve the same implicit equation with different inhomogeneous terms (Section 3.1).
//
// Mapping.  Cell (m, k) lies on anti-diagonal s = m + k and needs cells of s - 1 and s - 2 and
// the finished diagonal value of token m - 1, so all cells of one anti-diagonal are independent.
// One wavefront owns CP of the d_k + d_v columns of one chunk and keeps the whole sweep in
// registers: lane l holds the grid column k = l (and k = l + 64 for chunks beyond 64 tokens),
// whose value moves down one grid row per step while s - k runs from 1 to k.  The left neighbour
// Y(., k-1) is the next lower lane (a DPP wave rotate), its value of the step before is kept
// from the previous step, and the diagonal value Y(m-1, m-1) is the final value of lane m - 1,
// fetched with ds_bpermute.  No LDS storage, no barrier: the 2(C - 1) steps of the sweep are the
// only sequential dimension.  The r x r Gram coefficients come from a workspace that a Gram
// kernel (MFMA for bf16 inputs) fills first; they do not depend on the sweep and are prefetched
// one step ahead.
#include "pf_internal.h"
#include "pf_common.h"

namespace pf {

namespace {

template <typename T> __device__ __forceinline__ float ldf(const T *p);
template <> __device__ __forceinline__ float ldf<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ldf<uint16_t>(const uint16_t *p) { return bf16_bits_to_f32(*p); }

// ---- Gram of every chunk, plain version: one thread per entry.  Serves fp32 inputs and the
// shapes the MFMA version does not take.
template <typename T>
__global__ __launch_bounds__(256) void sigdelta_gram_plain(const T *__restrict__ K, const T *__restrict__ beta,
                                                          float *__restrict__ Gm, int L, int C, int NCt,
                                                          int dk, int r)
{
    const int chunk = blockIdx.x;                 // over heads * NCt
    const int head = chunk / NCt, c = chunk % NCt;
    const int cc = min(C, L - c * C), n = cc * r, np = C * r;
    const T *Kc = K + ((size_t)head * L + (size_t)c * C) * r * dk;
    const T *bc = beta + ((size_t)head * L + (size_t)c * C) * r;
    float *G = Gm + (size_t)chunk * np * np;
    for (int idx = blockIdx.y * blockDim.x + threadIdx.x; idx < n * n; idx += gridDim.y * blockDim.x) {
        const int row = idx / n, col = idx % n;
        if (row / r >= col / r) continue;         // only earlier tokens' rows are ever read
        const T *a = Kc + (size_t)row * dk, *b = Kc + (size_t)col * dk;
        float acc = 0.f;
        for (int e = 0; e < dk; ++e) acc = fmaf(ldf(a + e), ldf(b + e), acc);
        G[(size_t)row * np + col] = -ldf(bc + col) * acc;
    }
}

// ---- Gram of every chunk on MFMA (bf16 inputs, d_k a multiple of 32, C * r a multiple of 16):
// one wavefront per 16 x 16 tile of the upper triangle, both operands straight from global
// memory (a row's 8 consecutive elements are the A as well as the B operand slot of a lane).
__global__ __launch_bounds__(256) void sigdelta_gram_mfma(const bf16 *__restrict__ K, const bf16 *__restrict__ beta,
                                                         float *__restrict__ Gm, int L, int C, int NCt,
                                                         int dk, int r)
{
    const int chunk = blockIdx.x;
    const int head = chunk / NCt, c = chunk % NCt;
    const int cc = min(C, L - c * C), n = cc * r, np = C * r;
    const int NT = (n + 15) / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const bf16 *Kc = K + ((size_t)head * L + (size_t)c * C) * r * dk;
    const bf16 *bc = beta + ((size_t)head * L + (size_t)c * C) * r;
    float *G = Gm + (size_t)chunk * np * np;
    const int npairs = NT * (NT + 1) / 2;
    for (int p = blockIdx.y * 4 + wave; p < npairs; p += gridDim.y * 4) {
        int tj = 0, rem = p;                       // pair p -> (ti <= tj), column by column
        while (rem > tj) { rem -= tj + 1; ++tj; }
        const int ti = rem;
        const int ra = 16 * ti + r16, rb = 16 * tj + r16;
        const bf16 *pa = Kc + (size_t)min(ra, n - 1) * dk + 8 * g;
        const bf16 *pb = Kc + (size_t)min(rb, n - 1) * dk + 8 * g;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int kt = 0; kt < dk; kt += 32) acc = mfma16(ld8(pa + kt), ld8(pb + kt), acc);
        if (rb < n) {
            const float nb = -(float)bc[rb];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int row = 16 * ti + 4 * g + j;
                if (row < n) G[(size_t)row * np + rb] = nb * acc[j];
            }
        }
    }
}

// Full-wave rotate right by one lane (lane l receives lane l - 1, lane 0 receives lane 63).
__device__ __forceinline__ float wave_ror1(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x13C, 0xf, 0xf, false));
}
__device__ __forceinline__ float lane_fetch(float v, int src_lane)
{
    return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane << 2, __float_as_int(v)));
}

// ---- the sweep.  R rows per token, CP columns per wavefront, NS grid columns per lane.
template <typename T, int R, int CP, int NS>
__global__ __launch_bounds__(256) void sigdelta_sweep(const T *__restrict__ K, const T *__restrict__ V,
                                                      const T *__restrict__ beta, const float *__restrict__ Gm,
                                                      float *__restrict__ W, float *__restrict__ U,
                                                      int L, int C, int NCt, int dk, int dv, long long nwaves)
{
    const int lane = threadIdx.x & 63;
    const long long wv = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wv >= nwaves) return;                      // whole wavefronts only; no barrier below
    const int ngroups = (dk + dv) / CP;
    const int chunk = (int)(wv / ngroups), grp = (int)(wv % ngroups);
    const int head = chunk / NCt, c = chunk % NCt;
    const int cc = min(C, L - c * C), np = C * R;
    const size_t tok0 = (size_t)head * L + (size_t)c * C;
    const bool isW = grp * CP < dk;
    const int col0 = isW ? grp * CP : grp * CP - dk, dx = isW ? dk : dv;
    const T *X = (isW ? K : V) + tok0 * R * dx + col0;
    const T *bc = beta + tok0 * R;
    float *Y = (isW ? W : U) + tok0 * R * dx + col0;
    const float *G = Gm + (size_t)chunk * np * np;

    float cur[NS][R][CP], left2[NS][R][CP];
#pragma unroll
    for (int sl = 0; sl < NS; ++sl) {
        const int k = lane + 64 * sl;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const bool ok = k < cc;
            const float b = ok ? ldf(bc + k * R + j) : 0.f;
            const float sc = isW ? b : -b;         // A = beta k, Atil = -beta v
#pragma unroll
            for (int e = 0; e < CP; ++e) cur[sl][j][e] = ok ? sc * ldf(X + ((size_t)k * R + j) * dx + e) : 0.f;
        }
    }
    // left2 = left neighbour's grid row 0 (its value "two steps ago" as seen from step 1)
#pragma unroll
    for (int j = 0; j < R; ++j)
#pragma unroll
        for (int e = 0; e < CP; ++e) {
            const float r0 = wave_ror1(cur[0][j][e]);
            left2[0][j][e] = r0;
            if (NS == 2) {
                const float r1 = wave_ror1(cur[NS - 1][j][e]);
                left2[NS - 1][j][e] = lane == 0 ? r0 : r1;
            }
        }

    // coefficient of grid cell (m, k): rows (m-1, .) of the Gram, columns of token k minus
    // (off the diagonal) those of token k - 1; indices clamped where the cell does not exist
    auto load_coef = [&](int s, float (&cf)[NS][R][R]) {
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
            const int k = lane + 64 * sl, m = s - k;
            const bool act = m >= 1 && m <= k && k < cc;
            const int mm = act ? m - 1 : 0, kk = act ? k : 1;
            const bool offd = act && m < k;
#pragma unroll
            for (int jp = 0; jp < R; ++jp) {
                const float *row = G + (size_t)(mm * R + jp) * np;
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    const float hi = row[kk * R + j];
                    const float lo = offd ? row[(kk - 1) * R + j] : 0.f;
                    cf[sl][jp][j] = act ? hi - lo : 0.f;
                }
            }
        }
    };

    float cf[NS][R][R], cfn[NS][R][R];
    const int smax = 2 * (cc - 1);
    if (smax >= 1) load_coef(1, cf);
    for (int s = 1; s <= smax; ++s) {
        if (s < smax) load_coef(s + 1, cfn);
        bool act[NS], offd[NS];
        int src[NS];
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
            const int k = lane + 64 * sl, m = s - k;
            act[sl] = m >= 1 && m <= k && k < cc;
            offd[sl] = m < k;
            src[sl] = act[sl] ? m - 1 : 0;         // token whose finished value this cell needs
        }
#pragma unroll
        for (int e = 0; e < CP; ++e) {
            // every exchange reads the values of the step before; nothing of column e is
            // overwritten until all of them are in
            float l1[NS][R], dg[NS][R];
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const float r0 = wave_ror1(cur[0][j][e]);
                l1[0][j] = r0;
                dg[0][j] = lane_fetch(cur[0][j][e], src[0] & 63);
                if (NS == 2) {
                    const float r1 = wave_ror1(cur[NS - 1][j][e]);
                    l1[NS - 1][j] = lane == 0 ? r0 : r1;
                    const float d0 = lane_fetch(cur[0][j][e], src[NS - 1] & 63);
                    const float d1 = lane_fetch(cur[NS - 1][j][e], src[NS - 1] & 63);
                    dg[NS - 1][j] = src[NS - 1] >= 64 ? d1 : d0;
                }
            }
#pragma unroll
            for (int sl = 0; sl < NS; ++sl)
#pragma unroll
                for (int j = 0; j < R; ++j) {
                    const float own = cur[sl][j][e];
                    float acc = own + (offd[sl] ? l1[sl][j] - left2[sl][j][e] : 0.f);
#pragma unroll
                    for (int jp = 0; jp < R; ++jp) acc = fmaf(cf[sl][jp][j], dg[sl][jp], acc);
                    left2[sl][j][e] = l1[sl][j];
                    cur[sl][j][e] = act[sl] ? acc : own;
                }
        }
#pragma unroll
        for (int sl = 0; sl < NS; ++sl)
#pragma unroll
            for (int jp = 0; jp < R; ++jp)
#pragma unroll
                for (int j = 0; j < R; ++j) cf[sl][jp][j] = cfn[sl][jp][j];
    }

#pragma unroll
    for (int sl = 0; sl < NS; ++sl) {
        const int k = lane + 64 * sl;
        if (k < cc) {
#pragma unroll
            for (int j = 0; j < R; ++j)
#pragma unroll
                for (int e = 0; e < CP; e += 4) {
                    f32x4 v = {cur[sl][j][e], cur[sl][j][e + 1], cur[sl][j][e + 2], cur[sl][j][e + 3]};
                    *reinterpret_cast<f32x4 *>(Y + ((size_t)k * R + j) * dx + e) = v;
                }
        }
    }
}

template <typename T, int R, int CP, int NS>
hipError_t launch_sweep(const void *K, const void *V, const void *beta, const float *Gm, float *W, float *U,
                        int heads, int L, int C, int dk, int dv, hipStream_t stream)
{
    const int NCt = (L + C - 1) / C;
    const long long nwaves = (long long)heads * NCt * ((dk + dv) / CP);
    const long long blocks = (nwaves + 3) / 4;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((sigdelta_sweep<T, R, CP, NS>), dim3((unsigned)blocks), dim3(256), 0, stream,
                       static_cast<const T *>(K), static_cast<const T *>(V), static_cast<const T *>(beta), Gm, W, U,
                       L, C, NCt, dk, dv, nwaves);
    return hipGetLastError();
}

template <typename T>
hipError_t dispatch_sweep(const void *K, const void *V, const void *beta, const float *Gm, float *W, float *U,
                          int heads, int L, int C, int dk, int dv, int r, hipStream_t stream)
{
    const bool two = C > 64;
#define PF_SWEEP(R, CP1, CP2)                                                                                   \
    return two ? launch_sweep<T, R, CP2, 2>(K, V, beta, Gm, W, U, heads, L, C, dk, dv, stream)                \
               : launch_sweep<T, R, CP1, 1>(K, V, beta, Gm, W, U, heads, L, C, dk, dv, stream)
    switch (r) {
    case 1: PF_SWEEP(1, 16, 16);
    case 2: PF_SWEEP(2, 16, 16);
    case 4: PF_SWEEP(4, 16, 8);
    }
#undef PF_SWEEP
    return hipErrorInvalidValue;
}

}  // namespace

bool sigdelta_supported(int dk, int dv, int r, int chunk)
{
    return (r == 1 || r == 2 || r == 4) && chunk >= 1 && chunk <= 128 && dk % 16 == 0 && dv % 16 == 0;
}

size_t sigdelta_workspace_bytes(int heads, int L, int r, int chunk)
{
    const size_t NCt = ((size_t)L + chunk - 1) / chunk, np = (size_t)chunk * r;
    return (size_t)heads * NCt * np * np * sizeof(float);
}

hipError_t launch_sigdelta(const void *K, const void *V, const void *beta, float *W, float *U, float *Gm,
                           int heads, int L, int dk, int dv, int r, int chunk, bool is_bf16, hipStream_t stream)
{
    const int NCt = (L + chunk - 1) / chunk;
    const long long chunks = (long long)heads * NCt;
    if (chunks > 0x7fffffffLL) return hipErrorInvalidValue;
    const int np = chunk * r;
    if (is_bf16 && dk % 32 == 0 && np % 16 == 0) {
        const int NT = np / 16, npairs = NT * (NT + 1) / 2;
        hipLaunchKernelGGL(sigdelta_gram_mfma, dim3((unsigned)chunks, (unsigned)min((npairs + 3) / 4, 64)), dim3(256),
                           0, stream, static_cast<const bf16 *>(K), static_cast<const bf16 *>(beta), Gm, L, chunk,
                           NCt, dk, r);
    } else if (is_bf16) {
        hipLaunchKernelGGL((sigdelta_gram_plain<uint16_t>), dim3((unsigned)chunks, (unsigned)min((np * np + 255) / 256, 64)),
                           dim3(256), 0, stream, static_cast<const uint16_t *>(K),
                           static_cast<const uint16_t *>(beta), Gm, L, chunk, NCt, dk, r);
    } else {
        hipLaunchKernelGGL((sigdelta_gram_plain<float>), dim3((unsigned)chunks, (unsigned)min((np * np + 255) / 256, 64)),
                           dim3(256), 0, stream, static_cast<const float *>(K), static_cast<const float *>(beta),
                           Gm, L, chunk, NCt, dk, r);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return is_bf16 ? dispatch_sweep<uint16_t>(K, V, beta, Gm, W, U, heads, L, chunk, dk, dv, r, stream)
                   : dispatch_sweep<float>(K, V, beta, Gm, W, U, heads, L, chunk, dk, dv, r, stream);
}

}  // namespace pf
