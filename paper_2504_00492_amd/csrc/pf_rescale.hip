// beta -> beta_eff = (1 - exp(-beta |k|^2)) / |k|^2 for every (k, beta) pair: the step size with
// which a rank-1 delta step is the exact flow of its increment instead of its Euler step
// (Section 3.3 of ParallelFlow, arXiv 2504.00492: exp(a b^T) = Id + ((e^x - 1) / x) a b^T with
// x = <b, a>, here a = beta k, b = -k; the input increment picks up the same factor).
// One row of K per 16 lanes: 16-byte loads where the row length allows, partial sums combined
// with cross-lane shuffles (__shfl_xor) inside the 16-lane row, fp32 arithmetic.
#include "pf_internal.h"
#include "pf_common.h"

namespace pf {

namespace {

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<uint16_t>(uint16_t v) { return bf16_bits_to_f32(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ uint16_t from_f32<uint16_t>(float v)
{
    bf16 b = (bf16)v;
    return __builtin_bit_cast(uint16_t, b);
}

template <typename T>
__global__ __launch_bounds__(256) void beta_exponential_kernel(const T *__restrict__ K, const T *beta, T *beta_out,
                                                              long long rows, int dk)
{
    constexpr int VEC = 16 / sizeof(T);
    const int l16 = threadIdx.x & 15;
    const long long row0 = (long long)blockIdx.x * 16 + (threadIdx.x >> 4);
    for (long long row = row0; row < rows; row += (long long)gridDim.x * 16) {
        const T *k = K + row * dk;
        float s = 0.f;
        if (dk % VEC == 0) {
            for (int e = l16 * VEC; e < dk; e += 16 * VEC) {
                T v[VEC];
                *reinterpret_cast<u32x4 *>(v) = *reinterpret_cast<const u32x4 *>(k + e);
#pragma unroll
                for (int i = 0; i < VEC; ++i) s = fmaf(to_f32(v[i]), to_f32(v[i]), s);
            }
        } else {
            for (int e = l16; e < dk; e += 16) s = fmaf(to_f32(k[e]), to_f32(k[e]), s);
        }
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) s += __shfl_xor(s, m, 16);
        if (l16 == 0) {
            const float b = to_f32(beta[row]);
            const float be = s > 0.f ? -expm1f(-b * s) / s : b;
            beta_out[row] = from_f32<T>(be);
        }
    }
}

}  // namespace

hipError_t launch_beta_exponential(const void *K, const void *beta, void *beta_out, long long rows, int dk,
                                   bool is_bf16, hipStream_t stream)
{
    if (rows == 0) return hipSuccess;
    const long long want = (rows + 15) / 16;
    const unsigned grid = (unsigned)(want < 65536 ? want : 65536);
    if (is_bf16)
        hipLaunchKernelGGL(beta_exponential_kernel<uint16_t>, dim3(grid), dim3(256), 0, stream,
                           static_cast<const uint16_t *>(K), static_cast<const uint16_t *>(beta),
                           static_cast<uint16_t *>(beta_out), rows, dk);
    else
        hipLaunchKernelGGL(beta_exponential_kernel<float>, dim3(grid), dim3(256), 0, stream,
                           static_cast<const float *>(K), static_cast<const float *>(beta),
                           static_cast<float *>(beta_out), rows, dk);
    return hipGetLastError();
}

}  // namespace pf
