// Segment-parallel form of the state scan: step 3 of Section 3 of ParallelFlow (arXiv
// 2504.00492) as an actual scan over segments of the sequence instead of one hand-over chain
// per head, for workloads with too few heads to fill the GPU.
//
// The map of a segment (a run of consecutive flow blocks) on the state is affine,
//     S_out = S_in P_seg + H_seg,        P_seg in R^{d_k x d_k},  H_seg in R^{d_v x d_k},
// with P_seg the ordered product of the segment's transitions (Proposition 2.1) and H_seg what
// the segment writes into a zero state; affine maps compose, (P1, H1) then (P2, H2) =
// (P1 P2, H1 P2 + H2).  Rows of the state evolve independently, so both come out of the
// ordinary scan kernel: H_seg is its final state from S_0 = 0, and P_seg is its final state
// when the rows of the identity are fed in as the initial state and the values are zero.  The
// kernels here provide those two constants and the composition over the segments of a head;
// a last pass of the scan kernel then runs every segment from its true incoming state.
#include "pf_internal.h"
#include "pf_common.h"

namespace pf {

__global__ __launch_bounds__(256) void segment_constants_kernel(bf16 *zeroV, float *ident, int n, int d)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n * d) zeroV[i] = (bf16)0.0f;
    if (i < d * d) ident[i] = (i / d == i % d) ? 1.0f : 0.0f;
}

hipError_t launch_segment_constants(void *zeroV, float *ident, int n, int d, hipStream_t stream)
{
    const int m = n * d > d * d ? n * d : d * d;
    hipLaunchKernelGGL(segment_constants_kernel, dim3((m + 255) / 256), dim3(256), 0, stream,
                       (bf16 *)zeroV, ident, n, d);
    return hipGetLastError();
}

// One workgroup owns kRows rows of the state of one head (rows are independent) and walks the
// segments: S <- S P_s + H_s in fp32.  The rows live in LDS; a thread produces the columns
// x = tid, tid + 256, ... of every row.
constexpr int kComposeRows = 8;

__global__ __launch_bounds__(256) void segment_compose_kernel(const float *S0,
                                                              const float *__restrict__ Pseg,
                                                              const float *__restrict__ Hseg,
                                                              float *__restrict__ Sin, float *SL, int G, int d)
{
    extern __shared__ float rows[];                    // [2][kComposeRows][d]
    const int tiles = d / kComposeRows;
    const size_t head = blockIdx.x / tiles;
    const int r0 = (blockIdx.x % tiles) * kComposeRows;
    const int tid = threadIdx.x;
    float *cur = rows, *nxt = rows + kComposeRows * d;
    for (int i = tid; i < kComposeRows * d; i += 256)
        cur[i] = S0 ? S0[head * (size_t)d * d + (size_t)(r0 + i / d) * d + i % d] : 0.0f;
    __syncthreads();
    for (int s = 0; s < G; ++s) {
        const size_t seg = head * (size_t)G + s;
        for (int i = tid; i < kComposeRows * d; i += 256)
            Sin[seg * (size_t)d * d + (size_t)(r0 + i / d) * d + i % d] = cur[i];
        const float *P = Pseg + seg * (size_t)d * d;
        const float *H = Hseg + seg * (size_t)d * d;
        for (int x = tid; x < d; x += 256) {
            float acc[kComposeRows];
#pragma unroll
            for (int m = 0; m < kComposeRows; ++m) acc[m] = H[(size_t)(r0 + m) * d + x];
            for (int y = 0; y < d; ++y) {
                const float p = P[(size_t)y * d + x];   // coalesced over x
#pragma unroll
                for (int m = 0; m < kComposeRows; ++m) acc[m] = fmaf(cur[m * d + y], p, acc[m]);
            }
#pragma unroll
            for (int m = 0; m < kComposeRows; ++m) nxt[m * d + x] = acc[m];
        }
        __syncthreads();
        float *t = cur; cur = nxt; nxt = t;
    }
    if (SL)
        for (int i = tid; i < kComposeRows * d; i += 256)
            SL[head * (size_t)d * d + (size_t)(r0 + i / d) * d + i % d] = cur[i];
}

hipError_t launch_segment_compose(const float *S0, const float *Pseg, const float *Hseg, float *Sin,
                                  float *SL, int heads, int G, int d, hipStream_t stream)
{
    if (d % kComposeRows != 0) return hipErrorInvalidValue;
    const size_t lds = (size_t)2 * kComposeRows * d * sizeof(float);
    hipLaunchKernelGGL(segment_compose_kernel, dim3((unsigned)(heads * (d / kComposeRows))), dim3(256), lds,
                       stream, S0, Pseg, Hseg, Sin, SL, G, d);
    return hipGetLastError();
}

}  // namespace pf
