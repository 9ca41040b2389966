// C ABI of include/pf.h: argument checks on the host, then dispatch to the kernel launchers.
#include "../../include/pf.h"
#include "pf_internal.h"

namespace {

constexpr size_t kAlign = 256;
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Offsets (bytes) of the two per-chunk arrays inside the MFMA path's workspace.
struct WorkspacePlan {
    size_t oT, oP, total;
};
WorkspacePlan plan_workspace(int heads, int L, int d, int r, int chunk)
{
    (void)d;
    const size_t n = (size_t)chunk * r;
    const size_t tok = (size_t)heads * L;          // tokens over all heads
    const size_t tb = tok / chunk * n * n * 2;     // Tt: bf16, n*n per chunk
    const size_t pb = tok * n * 2;                 // Pt: bf16, chunk*n per chunk
    WorkspacePlan p;
    size_t o = 0;
    p.oT = o; o = round_up(o + tb, kAlign);
    p.oP = o; o = round_up(o + pb, kAlign);
    p.total = o;
    return p;
}

// Tokens per flow block on the MFMA path: the requested chunk, halved until chunk * r virtual
// tokens fit a kernel instance (the flow over a chunk is the composition of the flows over
// its halves, Section 3.1).  0 when no instance serves these dimensions.
int mfma_block(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (dt != PF_BF16 || d_k != d_v) return 0;
    for (int c = chunk; c >= 16; c /= 2) {
        if ((long long)c * r <= 4096 && pf::mfma_instance_exists(d_k, c * r, c)) return c;
        if (c % 2 != 0) break;
    }
    return 0;
}

int family(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (d_k <= 0 || d_v <= 0 || r <= 0 || chunk <= 0) return 0;
    if (dt != PF_F32 && dt != PF_BF16) return 0;
    if (mfma_block(d_k, d_v, r, chunk, dt) > 0) return 2;
    if ((long long)chunk * r > 65536 || d_k > 65536 || d_v > 65536) return 0;
    if (pf::generic_lds_bytes(d_k, d_v, r, chunk) <= pf::kMaxLdsBytes) return 1;
    return 0;
}

pf_status check_dims(int B, int H, int L, int d_k, int d_v, int r, int chunk)
{
    if (B <= 0 || H <= 0 || L < 0 || d_k <= 0 || d_v <= 0 || r <= 0 || chunk <= 0) return PF_ERR_SHAPE;
    if ((long long)B * H > 0x7fffffffLL) return PF_ERR_SHAPE;
    return PF_OK;
}

}  // namespace

extern "C" {

int pf_version(void) { return 100; }

const char *pf_status_str(pf_status s)
{
    switch (s) {
    case PF_OK: return "ok";
    case PF_ERR_NULL: return "a required pointer is NULL";
    case PF_ERR_SHAPE: return "bad dimension (non-positive, or L not a multiple of chunk on the MFMA path)";
    case PF_ERR_UNSUPPORTED: return "no kernel instance for these dimensions and dtype";
    case PF_ERR_ALIGN: return "a base address is not 16-byte aligned";
    case PF_ERR_WORKSPACE: return "workspace is NULL or too small";
    case PF_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    }
    return "unknown status";
}

int pf_delta_fwd_supported(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    return family(d_k, d_v, r, chunk, dt);
}

int pf_delta_fwd_block(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (d_k <= 0 || d_v <= 0 || r <= 0 || chunk <= 0) return 0;
    return mfma_block(d_k, d_v, r, chunk, dt);
}

size_t pf_delta_fwd_workspace_bytes(int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (check_dims(B, H, L, d_k, d_v, r, chunk) != PF_OK) return 0;
    if (family(d_k, d_v, r, chunk, dt) != 2 || L % chunk != 0) return 0;
    return plan_workspace(B * H, L, d_k, r, mfma_block(d_k, d_v, r, chunk, dt)).total;
}

pf_status pf_delta_fwd(const void *Q, const void *K, const void *V, const void *beta, const float *S0,
                       void *O, float *S_L, int B, int H, int L, int d_k, int d_v, int r, int chunk,
                       pf_dtype dt, void *workspace, size_t workspace_bytes, pf_stream stream)
{
    if (L != 0 && (!Q || !K || !V || !beta || !O)) return PF_ERR_NULL;
    pf_status st = check_dims(B, H, L, d_k, d_v, r, chunk);
    if (st != PF_OK) return st;
    int fam = family(d_k, d_v, r, chunk, dt);
    // The MFMA path needs whole chunks; a ragged L goes to the generic path when that fits.
    if (fam == 2 && L % chunk != 0)
        fam = (pf::generic_lds_bytes(d_k, d_v, r, chunk) <= pf::kMaxLdsBytes) ? 1 : -1;
    if (fam == -1) return PF_ERR_SHAPE;
    if (fam == 0) return PF_ERR_UNSUPPORTED;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(beta) || !aligned16(O) ||
        !aligned16(S0) || !aligned16(S_L))
        return PF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int heads = B * H;
    if (fam == 1 || L == 0) {
        hipError_t e = pf::launch_generic(Q, K, V, beta, S0, O, S_L, heads, L, d_k, d_v, r, chunk,
                                          dt == PF_BF16, s);
        return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
    }
    const int block = mfma_block(d_k, d_v, r, chunk, dt);
    const WorkspacePlan wp = plan_workspace(heads, L, d_k, r, block);
    if (!workspace || workspace_bytes < wp.total) return PF_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PF_ERR_ALIGN;
    char *ws = static_cast<char *>(workspace);
    hipError_t e = pf::launch_chunk_flow(Q, K, beta, ws + wp.oT, ws + wp.oP, heads, L, d_k, r, block, s);
    if (e != hipSuccess) return PF_ERR_LAUNCH;
    e = pf::launch_chunk_scan(Q, K, V, beta, ws + wp.oT, ws + wp.oP, S0, O, S_L, heads, L, d_k, r, block, s);
    return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
}

int pf_flow_fwd_supported(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (d_k <= 0 || d_v <= 0 || r <= 0 || chunk <= 0) return 0;
    if (dt != PF_F32 && dt != PF_BF16) return 0;
    if ((long long)chunk * r > 65536 || d_k > 65536 || d_v > 65536) return 0;
    return pf::generic_lds_bytes(d_k, d_v, r, chunk) <= pf::kMaxLdsBytes ? 1 : 0;
}

pf_status pf_flow_fwd(const void *Q, const void *A, const void *Atil, const void *Bm, const float *S0,
                      void *O, float *S_L, int B, int H, int L, int d_k, int d_v, int r, int chunk,
                      pf_dtype dt, pf_stream stream)
{
    if (L != 0 && (!Q || !A || !Atil || !Bm || !O)) return PF_ERR_NULL;
    pf_status st = check_dims(B, H, L, d_k, d_v, r, chunk);
    if (st != PF_OK) return st;
    if (!pf_flow_fwd_supported(d_k, d_v, r, chunk, dt)) return PF_ERR_UNSUPPORTED;
    if (!aligned16(Q) || !aligned16(A) || !aligned16(Atil) || !aligned16(Bm) || !aligned16(O) ||
        !aligned16(S0) || !aligned16(S_L))
        return PF_ERR_ALIGN;
    hipError_t e = pf::launch_generic_drivers(Q, A, Atil, Bm, S0, O, S_L, B * H, L, d_k, d_v, r, chunk,
                                              dt == PF_BF16, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
}

pf_status pf_delta_chunk_flow(const void *Q, const void *K, const void *beta, void *Tt, void *Pt,
                              int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_stream stream)
{
    if (!Q || !K || !beta || !Tt || !Pt) return PF_ERR_NULL;
    pf_status st = check_dims(B, H, L, d_k, d_v, r, chunk);
    if (st != PF_OK) return st;
    if (mfma_block(d_k, d_v, r, chunk, PF_BF16) != chunk) return PF_ERR_UNSUPPORTED;
    if (L % chunk != 0) return PF_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(beta) || !aligned16(Tt) || !aligned16(Pt))
        return PF_ERR_ALIGN;
    if (L == 0) return PF_OK;
    hipError_t e = pf::launch_chunk_flow(Q, K, beta, Tt, Pt, B * H, L, d_k, r, chunk,
                                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
}

pf_status pf_delta_chunk_scan(const void *Q, const void *K, const void *V, const void *beta, const void *Tt,
                              const void *Pt, const float *S0, void *O, float *S_L, int B, int H, int L,
                              int d_k, int d_v, int r, int chunk, pf_stream stream)
{
    if (!Q || !K || !V || !beta || !Tt || !Pt || !O) return PF_ERR_NULL;
    pf_status st = check_dims(B, H, L, d_k, d_v, r, chunk);
    if (st != PF_OK) return st;
    if (mfma_block(d_k, d_v, r, chunk, PF_BF16) != chunk) return PF_ERR_UNSUPPORTED;
    if (L % chunk != 0) return PF_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(beta) || !aligned16(Tt) ||
        !aligned16(Pt) || !aligned16(S0) || !aligned16(O) || !aligned16(S_L))
        return PF_ERR_ALIGN;
    hipError_t e = pf::launch_chunk_scan(Q, K, V, beta, Tt, Pt, S0, O, S_L, B * H, L, d_k, r, chunk,
                                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
}

}  // extern "C"
