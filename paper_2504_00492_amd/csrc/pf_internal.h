// Host-side launchers behind the C ABI of include/pf.h.  Each returns the HIP status of its
// launch; none of them allocates, frees or synchronises.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace pf {

constexpr size_t kMaxLdsBytes = 160 * 1024;  // LDS per workgroup (and per CU) on gfx950

// Compute units of the current device (asked once per device, then cached); 256, the count of
// an MI355X, when no device answers (host-only callers).
int device_cu_count();

// Opt a kernel in to `bytes` of dynamic LDS.  The attribute belongs to (kernel, device) and
// sticks, so it is set once per device: `armed` (one per kernel instantiation, zero-initialised)
// keeps a bit per device ordinal.
inline hipError_t arm_dynamic_lds(std::atomic<uint64_t> &armed, const void *kernel, size_t bytes)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = dev >= 0 && dev < 64 ? (uint64_t)1 << dev : 0;
    if (bit && (armed.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && bit) armed.fetch_or(bit, std::memory_order_release);
    return e;
}

// ---- generic path (pf_generic.hip)
size_t generic_lds_bytes(int dk, int dv, int r, int chunk);
// tokens [t0, L) of every head; the heads are L tokens apart in memory
hipError_t launch_generic(const void *Q, const void *K, const void *V, const void *beta, const float *S0,
                          void *O, float *SL, int heads, int L, int dk, int dv, int r, int chunk,
                          bool is_bf16, hipStream_t stream, int t0 = 0, bool product = false);
// (product: the r sub-updates of a token are applied one after another instead of as one additive
// rank-r increment; the solve mask is then strict in the virtual token.  Same flag below.)
// general drivers (A, Atil, B) of Section 3.1 through the same kernel
hipError_t launch_generic_drivers(const void *Q, const void *A, const void *Atil, const void *Bm,
                                  const float *S0, void *O, float *SL, int heads, int L, int dk, int dv,
                                  int r, int chunk, bool is_bf16, hipStream_t stream, int t0 = 0);

// ---- MFMA path (pf_flow.hip, pf_scan.hip); d = d_k = d_v, n = chunk * r.  Both launchers take
// the first L / chunk whole blocks of every head (heads L tokens apart) and leave the tail alone.
bool mfma_instance_exists(int d, int n, int chunk);
hipError_t launch_chunk_flow(const void *Q, const void *K, const void *beta, void *Tt, void *Pt,
                             int heads, int L, int d, int r, int chunk, hipStream_t stream,
                             bool product = false);
hipError_t launch_chunk_scan(const void *Q, const void *K, const void *V, const void *beta,
                             const void *Tt, const void *Pt, const float *S0, void *O, float *SL,
                             int heads, int L, int d, int r, int chunk, hipStream_t stream,
                             int vmul = 1, int s0mul = 1, int dv = 0);
// The same two kernels for the general drivers (A, Atil, B) of Section 3.1 (rows of A, B: d wide,
// of Atil: dv wide); instances with at most 128 virtual tokens per block.
bool mfma_general_instance_exists(int d, int n, int chunk);
hipError_t launch_chunk_flow_general(const void *Q, const void *A, const void *Bm, void *Tt, void *Pt, int heads,
                                     int L, int d, int r, int chunk, hipStream_t stream);
hipError_t launch_chunk_scan_general(const void *Q, const void *A, const void *Atil, const void *Bm, const void *Tt,
                                     const void *Pt, const float *S0, void *O, float *SL, int heads, int L, int d,
                                     int dv, int r, int chunk, hipStream_t stream);
// (O may be NULL: the state is advanced and S_L written, nothing is read out.  d = d_k; dv = d_v,
// a multiple of 16, 0 meaning d_v = d_k: V, O are dv wide and S0, S_L are dv x d.)
// d_v rows of S one scan workgroup owns for these dimensions (the scan runs heads * dv / tile chains)
int scan_dv_tile(int heads, int dv, int n);

// ---- fused forward (pf_fused.hip): flow and scan of every block in one kernel, d = d_k = d_v,
// n = chunk * r in {64, 128}.  Takes the first L / chunk whole blocks of every head.  Tdump / Pdump
// (may be NULL) receive T and P of every block in the layout of the split entry points.
bool fused_instance_exists(int d, int n, int chunk);
int fused_dv_tile(int heads, int d, int n, int chunk);
hipError_t launch_fused(const void *Q, const void *K, const void *V, const void *beta, const float *S0, void *O,
                        float *SL, void *Tdump, void *Pdump, int heads, int L, int d, int r, int chunk,
                        bool product, hipStream_t stream);

// ---- segment-parallel scan (pf_segments.hip): S0 / V constants and the composition of segments
// writes an n x d block of bf16 zeros at zeroV and the d x d fp32 identity at ident
hipError_t launch_segment_constants(void *zeroV, float *ident, int n, int d, hipStream_t stream);
// per head: Sin[0] = S0 (or 0); Sin[s+1] = Sin[s] Pseg[s] + Hseg[s]; S_L = Sin[G] (if not NULL)
hipError_t launch_segment_compose(const float *S0, const float *Pseg, const float *Hseg, float *Sin,
                                  float *SL, int heads, int G, int d, hipStream_t stream);

// ---- W, U of every chunk by the anti-diagonal sweep of Theorem 3.4 (pf_sigdelta.hip).  Gm is the
// Gram workspace of sigdelta_workspace_bytes(); the last chunk of a head may be short.
bool sigdelta_supported(int dk, int dv, int r, int chunk);
size_t sigdelta_workspace_bytes(int heads, int L, int r, int chunk);
hipError_t launch_sigdelta(const void *K, const void *V, const void *beta, float *W, float *U, float *Gm,
                           int heads, int L, int dk, int dv, int r, int chunk, bool is_bf16, hipStream_t stream);

// ---- exact rank-1 step size of Section 3.3 (pf_rescale.hip): one value per row of K
hipError_t launch_beta_exponential(const void *K, const void *beta, void *beta_out, long long rows, int dk,
                                   bool is_bf16, hipStream_t stream);

}  // namespace pf
