// C ABI of include/pf.h: argument checks on the host, then dispatch to the kernel launchers.
#include "../../include/pf.h"
#include "pf_internal.h"

#include <atomic>
#include <cstring>
#include <string>

namespace pf {

int device_cu_count()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cached[kMaxDevices];   // 0: not asked yet
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n > 0) return n;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
    cached[dev].store(n, std::memory_order_relaxed);
    return n;
}

}  // namespace pf

namespace {

constexpr size_t kAlign = 256;
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Offsets (bytes) of the two per-chunk arrays inside the MFMA path's workspace.
struct WorkspacePlan {
    size_t oT, oP, oS, oZ, oI, oH, oG, oSin, total;
    int segments;
};

// Segments per head for the segment-parallel scan: 1 (plain hand-over chain per head) unless
// the chains of the plain scan (heads x d_v tiles) would leave three quarters of the CUs idle
// and there are enough blocks to cut.  Three passes of the scan kernel then run with
// `segments` times as many chains.  Measured on 65536 tokens, d = 128, r = 2: eight segments
// on 4 heads 0.96 ms against 1.75 ms, four segments on 8 heads 1.52 against 1.83 ms; two
// segments (three passes over half the blocks each) cannot pay.
int scan_segments(int heads, int L, int d, int dv, int r, int chunk)
{
    if (L % chunk != 0 || d != dv) return 1;     // (the composition kernel takes square states)
    const int NC = L / chunk;
    const long long chains = (long long)heads * (d / pf::scan_dv_tile(heads, d, chunk * r));
    const int cus = pf::device_cu_count();
    if (chains > cus / 4 || NC < 32) return 1;
    int G = 1;
    while (2 * G * chains <= cus && NC % (2 * G) == 0 && NC / (2 * G) >= 4) G *= 2;
    return G >= 4 ? G : 1;
}
// L tokens per head of which the first L - L % chunk (whole flow blocks) go through the MFMA
// kernels; when a tail remains, a state buffer carries S from them to the kernel of the tail.
WorkspacePlan plan_workspace(int heads, int L, int d, int dv, int r, int chunk)
{
    const size_t n = (size_t)chunk * r;
    const size_t tok = (size_t)heads * (L - L % chunk);   // tokens in whole blocks over all heads
    const size_t tb = tok / chunk * n * n * 2;            // Tt: bf16, n*n per block
    const size_t pb = tok * n * 2;                        // Pt: bf16, chunk*n per block
    const size_t sb = L % chunk ? (size_t)heads * dv * d * 4 : 0;
    WorkspacePlan p;
    p.segments = scan_segments(heads, L, d, dv, r, chunk);
    const size_t gb = p.segments > 1 ? (size_t)heads * p.segments * d * d * 4 : 0;   // per-segment d x d fp32
    size_t o = 0;
    p.oT = o; o = round_up(o + tb, kAlign);
    p.oP = o; o = round_up(o + pb, kAlign);
    p.oS = o; o = round_up(o + sb, kAlign);
    p.oZ = o; o = round_up(o + (gb ? n * d * 2 : 0), kAlign);
    p.oI = o; o = round_up(o + (gb ? (size_t)d * d * 4 : 0), kAlign);
    p.oH = o; o = round_up(o + gb, kAlign);
    p.oG = o; o = round_up(o + gb, kAlign);
    p.oSin = o; o = round_up(o + gb, kAlign);
    p.total = o;
    return p;
}

// Tokens per chunk for the generic kernel when it takes the ragged tail of an MFMA-path call:
// the largest power of two up to 16 whose working set fits LDS next to the fp32 state (0: none).
int tail_chunk(int d, int dv, int r)
{
    for (int c = 16; c >= 1; c /= 2)
        if (pf::generic_lds_bytes(d, dv, r, c) <= pf::kMaxLdsBytes) return c;
    return 0;
}

// Tokens per flow block on the MFMA path: the requested chunk or chunk / 2^j (the flow over a
// chunk is the composition of the flows over its pieces, Section 3.1).  Small blocks are preferred
// where an instance exists: the hand-over array T grows with the square of the block and every d_v
// tile of a head reads all of it.  Measured (ms per forward; 64 / 128 / 256 virtual tokens per
// block): 64 heads x 4096 tokens, r = 2: 0.201 / 0.224 / -; 32 heads x 65536 tokens, r = 2:
// 2.31 / 2.39 / 3.27; r = 1, d = 64: 0.039 / 0.042 / -.  Blocks of fewer than 32 tokens lose again
// (r = 4: 16 tokens 0.542, 32 tokens 0.529, 64 tokens 0.752).  So: 64 virtual tokens if that is
// at least 32 tokens, else at most 128 virtual tokens, else the largest block that has an
// instance.  0 when no instance serves these dimensions.
template <typename Exists>
int pick_block(int r, int chunk, Exists exists)
{
    int any = 0, upto128 = 0;
    for (int c = chunk; c >= 16; c /= 2) {
        if ((long long)c * r <= 4096 && exists(c * r, c)) {
            if (c * r == 64 && c >= 32) return c;
            if (c * r <= 128 && !upto128) upto128 = c;
            if (!any) any = c;
        }
        if (c % 2 != 0) break;
    }
    return upto128 ? upto128 : any;
}

int mfma_block(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (dt != PF_BF16 || d_v % 16 != 0) return 0;   // d_k: where an instance exists (64, 128)
    return pick_block(r, chunk, [&](int n, int c) { return pf::mfma_instance_exists(d_k, n, c); });
}

// The same choice for the general drivers (measured: 64 heads x 4096 tokens, r = 2: 0.270 ms with
// blocks of 64 virtual tokens, 0.317 ms with 128); their instances end at 128 virtual tokens.
int mfma_general_block(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (dt != PF_BF16 || d_v % 16 != 0) return 0;
    return pick_block(r, chunk, [&](int n, int c) { return pf::mfma_general_instance_exists(d_k, n, c); });
}

// The split entry points take any (d, chunk * r, chunk) that has an instance.
bool split_instance(int d_k, int d_v, int r, int chunk)
{
    return d_v % 16 == 0 && (long long)chunk * r <= 4096 && pf::mfma_instance_exists(d_k, chunk * r, chunk);
}

// Tokens per chunk on the generic path: the requested chunk when its working set fits LDS next
// to the fp32 state, else the chunk halved until it does (the flow over a chunk is the composition
// of the flows over its pieces; the generic kernel takes a shorter last piece anyway).  0 when
// not even one token fits (the state alone is too large).
int generic_block(int d_k, int d_v, int r, int chunk)
{
    if (d_k > 65536 || d_v > 65536 || r > 65536) return 0;
    int c = chunk > 65536 / r ? 65536 / r : chunk;
    if (c < 1) return 0;
    while (c > 1 && pf::generic_lds_bytes(d_k, d_v, r, c) > pf::kMaxLdsBytes) c = (c + 1) / 2;
    return pf::generic_lds_bytes(d_k, d_v, r, c) <= pf::kMaxLdsBytes ? c : 0;
}

int family(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (d_k <= 0 || d_v <= 0 || r <= 0 || chunk <= 0) return 0;
    if (dt != PF_F32 && dt != PF_BF16) return 0;
    if (mfma_block(d_k, d_v, r, chunk, dt) > 0) return 2;
    return generic_block(d_k, d_v, r, chunk) > 0 ? 1 : 0;
}

pf_status check_dims(int B, int H, int L, int d_k, int d_v, int r, int chunk)
{
    if (B <= 0 || H <= 0 || L < 0 || d_k <= 0 || d_v <= 0 || r <= 0 || chunk <= 0) return PF_ERR_SHAPE;
    if ((long long)B * H > 0x7fffffffLL) return PF_ERR_SHAPE;
    return PF_OK;
}

// ---- scratch of pf_delta_fwd_static: a buffer inside the loaded code object, so that the entry
// point needs no allocation and no workspace argument.  In host code the array's name is only a
// stand-in for the symbol; its device address is asked once per device (each GPU holds its own
// copy at its own address) and only that pointer is ever passed on.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t static_scratch(void **out)
{
    constexpr int kMaxDevices = 64;
    static std::atomic<void *> cached[kMaxDevices];
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = cached[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        cached[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

}  // namespace

extern "C" {

int pf_version(void) { return 100; }

const char *pf_status_str(pf_status s)
{
    switch (s) {
    case PF_OK: return "ok";
    case PF_ERR_NULL: return "a required pointer is NULL";
    case PF_ERR_SHAPE: return "bad dimension (non-positive, or L not a multiple of chunk where that is required)";
    case PF_ERR_UNSUPPORTED: return "no kernel instance for these dimensions and dtype";
    case PF_ERR_ALIGN: return "a base address is not 16-byte aligned";
    case PF_ERR_WORKSPACE: return "workspace is NULL or too small";
    case PF_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    case PF_ERR_SCRATCH_LIMIT: return "the call needs more scratch than the library's static buffer holds";
    }
    return "unknown status";
}

int pf_delta_fwd_supported(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    return family(d_k, d_v, r, chunk, dt);
}

int pf_delta_fwd_block(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    const int fam = family(d_k, d_v, r, chunk, dt);
    if (fam == 2) return mfma_block(d_k, d_v, r, chunk, dt);
    return fam == 1 ? generic_block(d_k, d_v, r, chunk) : 0;
}

size_t pf_delta_fwd_workspace_bytes(int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (check_dims(B, H, L, d_k, d_v, r, chunk) != PF_OK) return 0;
    if (family(d_k, d_v, r, chunk, dt) != 2) return 0;
    const int block = mfma_block(d_k, d_v, r, chunk, dt);
    if (L < block) return 0;                         // all of it is tail: generic kernel, no scratch
    if (L % block != 0 && tail_chunk(d_k, d_v, r) == 0) return 0;
    return plan_workspace(B * H, L, d_k, d_v, r, block).total;
}

size_t pf_delta_fwd_describe(int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_dtype dt, char *buf,
                             size_t cap)
{
    std::string out;
    const int fam = check_dims(B, H, L, d_k, d_v, r, chunk) == PF_OK ? family(d_k, d_v, r, chunk, dt) : 0;
    if (fam != 0) {
        const char *elem = dt == PF_BF16 ? "unsigned short" : "float";
        const std::string generic = std::string("pf::generic_kernel<") + elem + ", false>";
        const int block = fam == 2 ? mfma_block(d_k, d_v, r, chunk, dt) : generic_block(d_k, d_v, r, chunk);
        const int tail = fam == 2 ? L % block : 0;
        if (fam == 1 || L < block) {
            out = generic;
        } else {
            const int heads = B * H, n = block * r;
            const int G = scan_segments(heads, L, d_k, d_v, r, block);
            const std::string dims = std::to_string(d_k) + ", " + std::to_string(n) + ", " + std::to_string(block);
            const std::string flow = "pf::flow_kernel<" + dims + ", false>";
            const std::string scan = "pf::scan_kernel<" + dims + ", " +
                                     std::to_string(pf::scan_dv_tile(heads * G, d_v, n));
            if (G > 1)
                out = flow + ";pf::segment_constants_kernel;" + scan + ", false, false>;" + scan + ", false, false>;" +
                      "pf::segment_compose_kernel;" + scan + ", true, false>";
            else
                out = flow + ";" + scan + ", true, false>";
            if (tail) out += ";" + generic;
        }
    }
    if (buf && cap > 0) {
        const size_t m = out.size() < cap - 1 ? out.size() : cap - 1;
        std::memcpy(buf, out.data(), m);
        buf[m] = '\0';
    }
    return out.size();
}

static pf_status delta_fwd_impl(const void *Q, const void *K, const void *V, const void *beta, const float *S0,
                                void *O, float *S_L, int B, int H, int L, int d_k, int d_v, int r, int chunk,
                                pf_dtype dt, void *workspace, size_t workspace_bytes, pf_stream stream,
                                bool product)
{
    if (L != 0 && (!Q || !K || !V || !beta || !O)) return PF_ERR_NULL;
    pf_status st = check_dims(B, H, L, d_k, d_v, r, chunk);
    if (st != PF_OK) return st;
    int fam = family(d_k, d_v, r, chunk, dt);
    if (fam == 0) return PF_ERR_UNSUPPORTED;
    // The MFMA kernels take whole flow blocks; the L % block tokens left over at the end of
    // every head go through the generic kernel, from the state the blocks leave behind.
    const int block = fam == 2 ? mfma_block(d_k, d_v, r, chunk, dt) : generic_block(d_k, d_v, r, chunk);
    const int tail = fam == 2 ? L % block : 0;
    const int tchunk = tail ? tail_chunk(d_k, d_v, r) : 0;
    if (tail && tchunk == 0) return PF_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(beta) || !aligned16(O) ||
        !aligned16(S0) || !aligned16(S_L))
        return PF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int heads = B * H;
    if (fam == 1 || L < block) {
        // generic family, an empty sequence, or a sequence shorter than one flow block
        hipError_t e = pf::launch_generic(Q, K, V, beta, S0, O, S_L, heads, L, d_k, d_v, r,
                                          fam == 1 ? block : (tchunk ? tchunk : 1), dt == PF_BF16, s, 0, product);
        return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
    }
    const WorkspacePlan wp = plan_workspace(heads, L, d_k, d_v, r, block);
    if (!workspace || workspace_bytes < wp.total) return PF_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PF_ERR_ALIGN;
    char *ws = static_cast<char *>(workspace);
    const float *state = S0;                       // state entering the tail
    {
        float *Smid = tail ? reinterpret_cast<float *>(ws + wp.oS) : S_L;
        const void *Tt = ws + wp.oT, *Pt = ws + wp.oP;
        hipError_t e = hipSuccess;
        if (wp.segments > 1) {
            e = pf::launch_chunk_flow(Q, K, beta, ws + wp.oT, ws + wp.oP, heads, L, d_k, r, block, s, product);
            if (e != hipSuccess) return PF_ERR_LAUNCH;
            // Segment-parallel scan (no tail here): every segment of every head is a chain of
            // its own.  What a segment does to a zero state, then its propagator (identity in,
            // zero values), then the composition over the segments of a head, then the real
            // pass of every segment from its true incoming state.
            const int G = wp.segments, vh = heads * G, Ls = L / G;
            float *Hseg = reinterpret_cast<float *>(ws + wp.oH), *Pseg = reinterpret_cast<float *>(ws + wp.oG);
            float *Sin = reinterpret_cast<float *>(ws + wp.oSin), *ident = reinterpret_cast<float *>(ws + wp.oI);
            e = pf::launch_segment_constants(ws + wp.oZ, ident, block * r, d_k, s);
            if (e != hipSuccess) return PF_ERR_LAUNCH;
            e = pf::launch_chunk_scan(Q, K, V, beta, Tt, Pt, nullptr, nullptr, Hseg, vh, Ls, d_k, r, block, s);
            if (e != hipSuccess) return PF_ERR_LAUNCH;
            e = pf::launch_chunk_scan(Q, K, ws + wp.oZ, beta, Tt, Pt, ident, nullptr, Pseg, vh, Ls, d_k, r, block, s, 0, 0);
            if (e != hipSuccess) return PF_ERR_LAUNCH;
            e = pf::launch_segment_compose(S0, Pseg, Hseg, Sin, S_L, heads, G, d_k, s);
            if (e != hipSuccess) return PF_ERR_LAUNCH;
            e = pf::launch_chunk_scan(Q, K, V, beta, Tt, Pt, Sin, O, nullptr, vh, Ls, d_k, r, block, s);
            return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
        } else {
            e = pf::launch_chunk_flow(Q, K, beta, ws + wp.oT, ws + wp.oP, heads, L, d_k, r, block, s, product);
            if (e != hipSuccess) return PF_ERR_LAUNCH;
            e = pf::launch_chunk_scan(Q, K, V, beta, Tt, Pt, S0, O, Smid, heads, L, d_k, r, block, s, 1, 1, d_v);
            if (e != hipSuccess) return PF_ERR_LAUNCH;
        }
        state = Smid;
    }
    if (tail) {
        hipError_t e = pf::launch_generic(Q, K, V, beta, state, O, S_L, heads, L, d_k, d_v, r, tchunk, true, s,
                                          L - tail, product);
        if (e != hipSuccess) return PF_ERR_LAUNCH;
    }
    return PF_OK;
}

pf_status pf_delta_fwd(const void *Q, const void *K, const void *V, const void *beta, const float *S0,
                       void *O, float *S_L, int B, int H, int L, int d_k, int d_v, int r, int chunk,
                       pf_dtype dt, void *workspace, size_t workspace_bytes, pf_stream stream)
{
    return delta_fwd_impl(Q, K, V, beta, S0, O, S_L, B, H, L, d_k, d_v, r, chunk, dt, workspace, workspace_bytes,
                          stream, false);
}

pf_status pf_delta_product_fwd(const void *Q, const void *K, const void *V, const void *beta, const float *S0,
                               void *O, float *S_L, int B, int H, int L, int d_k, int d_v, int r, int chunk,
                               pf_dtype dt, void *workspace, size_t workspace_bytes, pf_stream stream)
{
    return delta_fwd_impl(Q, K, V, beta, S0, O, S_L, B, H, L, d_k, d_v, r, chunk, dt, workspace, workspace_bytes,
                          stream, true);
}

pf_status pf_init(void)
{
    void *p = nullptr;
    if (static_scratch(&p) != hipSuccess) return PF_ERR_LAUNCH;
    (void)pf::device_cu_count();
    return PF_OK;
}

size_t pf_delta_fwd_static_limit(void) { return kStaticScratchBytes; }

pf_status pf_delta_fwd_static(const void *Q, const void *K, const void *V, const void *beta, const float *S0,
                              void *O, float *S_L, int B, int H, int L, int d_k, int d_v, int r, int chunk,
                              pf_dtype dt, pf_stream stream)
{
    // every check that needs no device first, so that a bad call has no effect at all
    if (L != 0 && (!Q || !K || !V || !beta || !O)) return PF_ERR_NULL;
    pf_status st = check_dims(B, H, L, d_k, d_v, r, chunk);
    if (st != PF_OK) return st;
    if (family(d_k, d_v, r, chunk, dt) == 0) return PF_ERR_UNSUPPORTED;
    const size_t need = pf_delta_fwd_workspace_bytes(B, H, L, d_k, d_v, r, chunk, dt);
    if (need > kStaticScratchBytes) return PF_ERR_SCRATCH_LIMIT;
    void *ws = nullptr;
    if (need > 0 && static_scratch(&ws) != hipSuccess) return PF_ERR_LAUNCH;
    // Nothing in the scratch has to start at zero: every tile of T and P that the scan kernel
    // reads is written by the flow kernel of the same call, and the segment-parallel path
    // writes its constants itself.  What an earlier call left behind is simply overwritten.
    return delta_fwd_impl(Q, K, V, beta, S0, O, S_L, B, H, L, d_k, d_v, r, chunk, dt, ws, need ? kStaticScratchBytes : 0,
                          stream, false);
}

int pf_delta_fwd_fused_supported(int d_k, int d_v, int r, int chunk)
{
    if (d_k <= 0 || d_v <= 0 || r <= 0 || chunk <= 0 || d_k != d_v || (long long)chunk * r > 4096) return 0;
    return pf::fused_instance_exists(d_k, chunk * r, chunk) ? 1 : 0;
}

pf_status pf_delta_fwd_fused(const void *Q, const void *K, const void *V, const void *beta, const float *S0,
                             void *O, float *S_L, int B, int H, int L, int d_k, int d_v, int r, int chunk,
                             int product, pf_stream stream)
{
    if (L != 0 && (!Q || !K || !V || !beta || !O)) return PF_ERR_NULL;
    pf_status st = check_dims(B, H, L, d_k, d_v, r, chunk);
    if (st != PF_OK) return st;
    if (!pf_delta_fwd_fused_supported(d_k, d_v, r, chunk)) return PF_ERR_UNSUPPORTED;
    if (L % chunk != 0) return PF_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(beta) || !aligned16(O) ||
        !aligned16(S0) || !aligned16(S_L))
        return PF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (L == 0) {
        // nothing to scan: the generic launcher copies the state through
        hipError_t e = pf::launch_generic(Q, K, V, beta, S0, O, S_L, B * H, 0, d_k, d_v, r, 1, true, s, 0,
                                          product != 0);
        return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
    }
    hipError_t e = pf::launch_fused(Q, K, V, beta, S0, O, S_L, nullptr, nullptr, B * H, L, d_k, r, chunk,
                                    product != 0, s);
    return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
}

int pf_flow_fwd_supported(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (d_k <= 0 || d_v <= 0 || r <= 0 || chunk <= 0) return 0;
    if (dt != PF_F32 && dt != PF_BF16) return 0;
    return generic_block(d_k, d_v, r, chunk) > 0 ? 1 : 0;
}

int pf_flow_fwd_mfma_block(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (d_k <= 0 || d_v <= 0 || r <= 0 || chunk <= 0) return 0;
    return mfma_general_block(d_k, d_v, r, chunk, dt);
}

size_t pf_flow_fwd_mfma_workspace_bytes(int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (check_dims(B, H, L, d_k, d_v, r, chunk) != PF_OK) return 0;
    const int block = pf_flow_fwd_mfma_block(d_k, d_v, r, chunk, dt);
    if (block == 0 || L < block) return 0;
    const size_t n = (size_t)block * r, heads = (size_t)B * H;
    const size_t tok = heads * (L - L % block);
    size_t o = round_up(tok / block * n * n * 2, kAlign);          // T of every block
    o = round_up(o + tok * n * 2, kAlign);                         // P of every block
    if (L % block) o = round_up(o + heads * d_v * d_k * 4, kAlign);   // the state handed to the tail
    return o;
}

pf_status pf_flow_fwd_mfma(const void *Q, const void *A, const void *Atil, const void *Bm, const float *S0,
                           void *O, float *S_L, int B, int H, int L, int d_k, int d_v, int r, int chunk,
                           pf_dtype dt, void *workspace, size_t workspace_bytes, pf_stream stream)
{
    if (L != 0 && (!Q || !A || !Atil || !Bm || !O)) return PF_ERR_NULL;
    pf_status st = check_dims(B, H, L, d_k, d_v, r, chunk);
    if (st != PF_OK) return st;
    const int block = pf_flow_fwd_mfma_block(d_k, d_v, r, chunk, dt);
    if (block == 0) return PF_ERR_UNSUPPORTED;
    const int tail = L % block;
    const int tchunk = tail_chunk(d_k, d_v, r);
    if ((tail || L < block) && tchunk == 0) return PF_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(A) || !aligned16(Atil) || !aligned16(Bm) || !aligned16(O) ||
        !aligned16(S0) || !aligned16(S_L))
        return PF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int heads = B * H;
    if (L < block) {
        hipError_t e = pf::launch_generic_drivers(Q, A, Atil, Bm, S0, O, S_L, heads, L, d_k, d_v, r, tchunk, true, s);
        return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
    }
    const size_t need = pf_flow_fwd_mfma_workspace_bytes(B, H, L, d_k, d_v, r, chunk, dt);
    if (!workspace || workspace_bytes < need) return PF_ERR_WORKSPACE;
    if (!aligned16(workspace)) return PF_ERR_ALIGN;
    char *ws = static_cast<char *>(workspace);
    const size_t n = (size_t)block * r, tok = (size_t)heads * (L - tail);
    char *Tt = ws, *Pt = ws + round_up(tok / block * n * n * 2, kAlign);
    float *Smid = tail ? reinterpret_cast<float *>(Pt + round_up(tok * n * 2, kAlign)) : S_L;
    hipError_t e = pf::launch_chunk_flow_general(Q, A, Bm, Tt, Pt, heads, L, d_k, r, block, s);
    if (e != hipSuccess) return PF_ERR_LAUNCH;
    e = pf::launch_chunk_scan_general(Q, A, Atil, Bm, Tt, Pt, S0, O, Smid, heads, L, d_k, d_v, r, block, s);
    if (e != hipSuccess) return PF_ERR_LAUNCH;
    if (tail) {
        e = pf::launch_generic_drivers(Q, A, Atil, Bm, Smid, O, S_L, heads, L, d_k, d_v, r, tchunk, true, s, L - tail);
        if (e != hipSuccess) return PF_ERR_LAUNCH;
    }
    return PF_OK;
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
    hipError_t e = pf::launch_generic_drivers(Q, A, Atil, Bm, S0, O, S_L, B * H, L, d_k, d_v, r,
                                              generic_block(d_k, d_v, r, chunk), dt == PF_BF16,
                                              static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
}

int pf_delta_chunk_supported(int d_k, int d_v, int r, int chunk)
{
    if (d_k <= 0 || d_v <= 0 || r <= 0 || chunk <= 0) return 0;
    return split_instance(d_k, d_v, r, chunk) ? 1 : 0;
}

pf_status pf_delta_chunk_flow(const void *Q, const void *K, const void *beta, void *Tt, void *Pt,
                              int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_stream stream)
{
    if (!Q || !K || !beta || !Tt || !Pt) return PF_ERR_NULL;
    pf_status st = check_dims(B, H, L, d_k, d_v, r, chunk);
    if (st != PF_OK) return st;
    if (!split_instance(d_k, d_v, r, chunk)) return PF_ERR_UNSUPPORTED;
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
    if (!split_instance(d_k, d_v, r, chunk)) return PF_ERR_UNSUPPORTED;
    if (L % chunk != 0) return PF_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(beta) || !aligned16(Tt) ||
        !aligned16(Pt) || !aligned16(S0) || !aligned16(O) || !aligned16(S_L))
        return PF_ERR_ALIGN;
    hipError_t e = pf::launch_chunk_scan(Q, K, V, beta, Tt, Pt, S0, O, S_L, B * H, L, d_k, r, chunk,
                                         static_cast<hipStream_t>(stream), 1, 1, d_v);
    return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
}

pf_status pf_beta_exponential(const void *K, const void *beta, void *beta_out, int B, int H, int L, int d_k,
                              int r, pf_dtype dt, pf_stream stream)
{
    if (L != 0 && (!K || !beta || !beta_out)) return PF_ERR_NULL;
    if (B <= 0 || H <= 0 || L < 0 || d_k <= 0 || r <= 0 || (long long)B * H > 0x7fffffffLL) return PF_ERR_SHAPE;
    if (dt != PF_F32 && dt != PF_BF16) return PF_ERR_UNSUPPORTED;
    if (!aligned16(K) || !aligned16(beta) || !aligned16(beta_out)) return PF_ERR_ALIGN;
    hipError_t e = pf::launch_beta_exponential(K, beta, beta_out, (long long)B * H * L * r, d_k, dt == PF_BF16,
                                               static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
}

int pf_delta_chunk_sigdelta_supported(int d_k, int d_v, int r, int chunk, pf_dtype dt)
{
    if (d_k <= 0 || d_v <= 0 || r <= 0 || chunk <= 0) return 0;
    if (dt != PF_F32 && dt != PF_BF16) return 0;
    return pf::sigdelta_supported(d_k, d_v, r, chunk) ? 1 : 0;
}

size_t pf_delta_chunk_sigdelta_workspace_bytes(int B, int H, int L, int r, int chunk)
{
    if (B <= 0 || H <= 0 || L <= 0 || r <= 0 || chunk <= 0 || (long long)B * H > 0x7fffffffLL) return 0;
    return pf::sigdelta_workspace_bytes(B * H, L, r, chunk);
}

pf_status pf_delta_chunk_sigdelta(const void *K, const void *V, const void *beta, float *W, float *U,
                                  int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_dtype dt,
                                  void *workspace, size_t workspace_bytes, pf_stream stream)
{
    if (L != 0 && (!K || !V || !beta || !W || !U)) return PF_ERR_NULL;
    pf_status st = check_dims(B, H, L, d_k, d_v, r, chunk);
    if (st != PF_OK) return st;
    if (!pf_delta_chunk_sigdelta_supported(d_k, d_v, r, chunk, dt)) return PF_ERR_UNSUPPORTED;
    if (L == 0) return PF_OK;
    if (!workspace || workspace_bytes < pf::sigdelta_workspace_bytes(B * H, L, r, chunk)) return PF_ERR_WORKSPACE;
    if (!aligned16(K) || !aligned16(V) || !aligned16(beta) || !aligned16(W) || !aligned16(U) ||
        !aligned16(workspace))
        return PF_ERR_ALIGN;
    hipError_t e = pf::launch_sigdelta(K, V, beta, W, U, static_cast<float *>(workspace), B * H, L, d_k, d_v, r,
                                       chunk, dt == PF_BF16, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PF_OK : PF_ERR_LAUNCH;
}

}  // extern "C"
