// Generic path: one workgroup per (b, h), fp32 vector arithmetic, the chunk's working set in
// LDS.  Serves PF_F32 and every shape the MFMA path has no instance for (any d_k, d_v, r,
// chunk that fits LDS; a shorter last chunk when L is not a multiple of chunk).
//
// Per chunk it takes the steps of Theorem 3.2 (ParallelFlow, arXiv 2504.00492) in delta
// variables, n = (tokens in chunk) * r virtual tokens:
//   G      = M (.) diag(beta) K K^T          M strict in time               (system matrix - Id)
//   [W|U'] = (Id + G)^{-1} [beta K | beta V]  by forward substitution, token by token
//            (Proposition 3.3; the r rows of one token do not see each other)
//   U_eff  = U' - W S^T                      (U + W S_0^T of Theorem 3.2)
//   O      = Q S^T + (Mbar (.) Q K^T) U_eff   Mbar inclusive in time       (flow truncated at t)
//   S     += U_eff^T K                       (S_1 of Theorem 3.2)
//
// The same kernel serves the general low-rank drivers of Section 3.1,
//   S_t = S_{t-1} + S_{t-1} A_t B_t^T + Atil_t B_t^T,
// by loading (K, beta K, beta V) := (-B, A, -Atil): Theorem 3.2's Id - M (.) A B^T is then
// Id + M (.) (A)(-B)^T, its U + W S_0^T is -(U_eff), and every later line is unchanged.
#include "pf_internal.h"
#include "pf_common.h"

namespace pf {

template <typename T> __device__ __forceinline__ float load_as_f32(const T *p, size_t i);
template <> __device__ __forceinline__ float load_as_f32<float>(const float *p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float load_as_f32<uint16_t>(const uint16_t *p, size_t i)
{
    return bf16_bits_to_f32(p[i]);
}
template <typename T> __device__ __forceinline__ void store_from_f32(T *p, size_t i, float v);
template <> __device__ __forceinline__ void store_from_f32<float>(float *p, size_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void store_from_f32<uint16_t>(uint16_t *p, size_t i, float v)
{
    bf16 b = (bf16)v;
    p[i] = __builtin_bit_cast(uint16_t, b);
}

// LDS plan (floats), identical on host and device.
struct GenericPlan {
    int ldk, ldv, ldn;          // padded row pitches
    size_t oS, oK, oW, oU, oQ, oG, oP, total;
};
__host__ __device__ inline GenericPlan generic_plan(int dk, int dv, int r, int chunk)
{
    GenericPlan p;
    const int n = chunk * r;
    p.ldk = dk + 1; p.ldv = dv + 1; p.ldn = n + 1;
    size_t o = 0;
    p.oS = o; o += (size_t)dv * p.ldk;
    p.oK = o; o += (size_t)n * p.ldk;
    p.oW = o; o += (size_t)n * p.ldk;
    p.oU = o; o += (size_t)n * p.ldv;
    p.oQ = o; o += (size_t)chunk * p.ldk;
    p.oG = o; o += (size_t)n * p.ldn;
    p.oP = o; o += (size_t)chunk * p.ldn;
    p.total = o;
    return p;
}

// rs = rows of the system that are solved together and do not see each other: r for the paper's
// additive rank-r increment (Theorem 3.2's mask, strict in time), 1 for the product form, in
// which the r sub-updates of a token are applied one after another (mask strict in the virtual
// token).  The readout mask is the same in both.
// kDrivers == false: (K, V, beta) are keys, values, betas of the delta rule.
// kDrivers == true:  (K, V, beta) are (B, Atil, A) of the general recurrence (beta: [.., r, d_k]).
template <typename T, bool kDrivers>
__global__ __launch_bounds__(256) void generic_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                      const T *__restrict__ V, const T *__restrict__ beta,
                                                      const float *S0, T *__restrict__ O, float *SL,
                                                      int L, int dk, int dv, int r, int chunk, int t0,
                                                      int rs)
{
    extern __shared__ float smem[];
    const GenericPlan pl = generic_plan(dk, dv, r, chunk);
    float *S = smem + pl.oS, *Kc = smem + pl.oK, *Wc = smem + pl.oW, *Uc = smem + pl.oU;
    float *Qc = smem + pl.oQ, *G = smem + pl.oG, *Pm = smem + pl.oP;
    const int ldk = pl.ldk, ldv = pl.ldv, ldn = pl.ldn;
    const int tid = threadIdx.x, nth = blockDim.x;
    const size_t head = blockIdx.x;
    const T *Qh = Q + head * (size_t)L * dk;
    const T *Kh = K + head * (size_t)L * r * dk;
    const T *Vh = V + head * (size_t)L * r * dv;
    const T *bh = beta + head * (size_t)L * r * (kDrivers ? dk : 1);
    T *Oh = O + head * (size_t)L * dv;

    for (int i = tid; i < dv * dk; i += nth) {
        const int m = i / dk, x = i % dk;
        S[m * ldk + x] = S0 ? S0[head * (size_t)dv * dk + i] : 0.0f;
    }
    __syncthreads();

    for (int c0 = t0; c0 < L; c0 += chunk) {   // tokens before t0 belong to another kernel
        const int cl = min(chunk, L - c0);   // tokens in this chunk (shorter tail allowed)
        const int n = cl * r;                // virtual tokens in this chunk
        // ---- load: K, W = beta K, U = beta V, Q
        for (int i = tid; i < n * dk; i += nth) {
            const int row = i / dk, x = i % dk;
            const float kv = load_as_f32(Kh, ((size_t)c0 * r + row) * dk + x);
            if (kDrivers) {
                Kc[row * ldk + x] = -kv;
                Wc[row * ldk + x] = load_as_f32(bh, ((size_t)c0 * r + row) * dk + x);
            } else {
                Kc[row * ldk + x] = kv;
                Wc[row * ldk + x] = load_as_f32(bh, (size_t)c0 * r + row) * kv;
            }
        }
        for (int i = tid; i < n * dv; i += nth) {
            const int row = i / dv, m = i % dv;
            const float vv = load_as_f32(Vh, ((size_t)c0 * r + row) * dv + m);
            Uc[row * ldv + m] = kDrivers ? -vv : load_as_f32(bh, (size_t)c0 * r + row) * vv;
        }
        for (int i = tid; i < cl * dk; i += nth) {
            const int t = i / dk, x = i % dk;
            Qc[t * ldk + x] = load_as_f32(Qh, ((size_t)c0 + t) * dk + x);
        }
        __syncthreads();
        // ---- G = M (.) (beta K) K^T  and  P = Mbar (.) Q K^T   (W still holds beta K here)
        for (int i = tid; i < n * n; i += nth) {
            const int row = i / n, col = i % n;
            float acc = 0.0f;
            if (col / rs < row / rs)
                for (int x = 0; x < dk; ++x) acc = fmaf(Wc[row * ldk + x], Kc[col * ldk + x], acc);
            G[row * ldn + col] = acc;
        }
        for (int i = tid; i < cl * n; i += nth) {
            const int t = i / n, col = i % n;
            float acc = 0.0f;
            if (col / r <= t)
                for (int x = 0; x < dk; ++x) acc = fmaf(Qc[t * ldk + x], Kc[col * ldk + x], acc);
            Pm[t * ldn + col] = acc;
        }
        __syncthreads();
        // ---- forward substitution, rs rows at a time (one token, or one virtual token)
        const int ncol = dk + dv;
        for (int t = 1; t < n / rs; ++t) {
            for (int i = tid; i < rs * ncol; i += nth) {
                const int row = t * rs + i / ncol, col = i % ncol;
                float acc = 0.0f;
                if (col < dk) {
                    for (int j = 0; j < t * rs; ++j) acc = fmaf(G[row * ldn + j], Wc[j * ldk + col], acc);
                    Wc[row * ldk + col] -= acc;
                } else {
                    const int m = col - dk;
                    for (int j = 0; j < t * rs; ++j) acc = fmaf(G[row * ldn + j], Uc[j * ldv + m], acc);
                    Uc[row * ldv + m] -= acc;
                }
            }
            __syncthreads();
        }
        // ---- U_eff = U' - W S^T
        for (int i = tid; i < n * dv; i += nth) {
            const int row = i / dv, m = i % dv;
            float acc = 0.0f;
            for (int x = 0; x < dk; ++x) acc = fmaf(Wc[row * ldk + x], S[m * ldk + x], acc);
            Uc[row * ldv + m] -= acc;
        }
        __syncthreads();
        // ---- O = Q S^T + P U_eff
        for (int i = tid; i < cl * dv; i += nth) {
            const int t = i / dv, m = i % dv;
            float acc = 0.0f;
            for (int x = 0; x < dk; ++x) acc = fmaf(Qc[t * ldk + x], S[m * ldk + x], acc);
            for (int j = 0; j < (t + 1) * r; ++j) acc = fmaf(Pm[t * ldn + j], Uc[j * ldv + m], acc);
            store_from_f32(Oh, ((size_t)c0 + t) * dv + m, acc);
        }
        __syncthreads();
        // ---- S += U_eff^T K
        for (int i = tid; i < dv * dk; i += nth) {
            const int m = i / dk, x = i % dk;
            float acc = S[m * ldk + x];
            for (int j = 0; j < n; ++j) acc = fmaf(Uc[j * ldv + m], Kc[j * ldk + x], acc);
            S[m * ldk + x] = acc;
        }
        __syncthreads();
    }
    if (SL)
        for (int i = tid; i < dv * dk; i += nth) SL[head * (size_t)dv * dk + i] = S[(i / dk) * ldk + i % dk];
}

size_t generic_lds_bytes(int dk, int dv, int r, int chunk)
{
    return generic_plan(dk, dv, r, chunk).total * sizeof(float);
}

template <typename T, bool kDrivers>
static hipError_t launch_generic_instance(const void *Q, const void *K, const void *V, const void *beta,
                                          const float *S0, void *O, float *SL, int heads, int L, int dk, int dv,
                                          int r, int chunk, int t0, bool product, hipStream_t stream)
{
    const size_t lds = generic_lds_bytes(dk, dv, r, chunk);
    auto kern = generic_kernel<T, kDrivers>;
    // the opt-in is for the largest size any call may ask for, so that it is made once per device
    static std::atomic<uint64_t> armed{0};
    hipError_t e = arm_dynamic_lds(armed, reinterpret_cast<const void *>(kern), kMaxLdsBytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(heads), dim3(256), lds, stream, (const T *)Q, (const T *)K, (const T *)V,
                       (const T *)beta, S0, (T *)O, SL, L, dk, dv, r, chunk, t0, product ? 1 : r);
    return hipGetLastError();
}

hipError_t launch_generic(const void *Q, const void *K, const void *V, const void *beta, const float *S0,
                          void *O, float *SL, int heads, int L, int dk, int dv, int r, int chunk,
                          bool is_bf16, hipStream_t stream, int t0, bool product)
{
    return is_bf16 ? launch_generic_instance<uint16_t, false>(Q, K, V, beta, S0, O, SL, heads, L, dk, dv, r, chunk, t0, product, stream)
                   : launch_generic_instance<float, false>(Q, K, V, beta, S0, O, SL, heads, L, dk, dv, r, chunk, t0, product, stream);
}

hipError_t launch_generic_drivers(const void *Q, const void *A, const void *Atil, const void *Bm, const float *S0,
                                  void *O, float *SL, int heads, int L, int dk, int dv, int r, int chunk,
                                  bool is_bf16, hipStream_t stream, int t0)
{
    return is_bf16 ? launch_generic_instance<uint16_t, true>(Q, Bm, Atil, A, S0, O, SL, heads, L, dk, dv, r, chunk, t0, false, stream)
                   : launch_generic_instance<float, true>(Q, Bm, Atil, A, S0, O, SL, heads, L, dk, dv, r, chunk, t0, false, stream);
}

}  // namespace pf
