/*
 * pf.h - C ABI of the MI355X (gfx950) chunked forward of the low-rank delta rule
 *        (ParallelFlow, arXiv 2504.00492).
 *
 * The operation (one independent recurrence per (b, h)):
 *
 *     S_t = S_{t-1} (I - sum_j beta_{t,j} k_{t,j} k_{t,j}^T) + sum_j beta_{t,j} v_{t,j} k_{t,j}^T
 *     o_t = S_t q_t                          t = 0 .. L-1,  j = 0 .. r-1,  S in R^{d_v x d_k}
 *
 * i.e. the discretised dynamics of Section 3.1 under the delta mapping of the Remark in
 * Section 3.1 (A = beta k, Atil = -beta v, B = -k; rank r = one additive rank-r increment
 * per token), with the "memory readout" of Section 1.1 on the updated state.  For r = 1 this
 * is the DeltaNet update of Section 1.3.  It is computed chunk by chunk as the flow of the
 * system (Section 3): per chunk the compact form of Theorem 3.2 (W = T beta K, U = -T beta V with
 * T the inverse of the chunk's triangular system matrix, obtained by the block substitution
 * of Proposition 3.3); the readout inside the chunk from the same T; and a state hand-over from
 * chunk to chunk.
 *
 * Conventions common to every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees or synchronises; work is enqueued on `stream` and returns at once.
 *   - Tensors are dense, row-major, innermost dimension contiguous, base addresses 16-byte
 *     aligned (PF_ERR_ALIGN otherwise).
 *   - `dt` is the element type of Q, K, V, beta and O.  S0, S_L are always fp32.  All
 *     accumulation is fp32; for PF_BF16 the MFMA operands are bf16.
 *   - beta is used as given (any real value); keys are not normalised; q is not scaled.
 *   - Errors are return codes; nothing is printed, thrown or aborted.  Every argument check
 *     happens on the host before anything is launched, so a failing call has no effect.
 *   - Calls that share a workspace (or outputs) must be ordered by the caller (same stream).
 */
#ifndef PF_H
#define PF_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PF_OK = 0,
    PF_ERR_NULL = 1,        /* a required pointer is NULL */
    PF_ERR_SHAPE = 2,       /* a dimension is <= 0, or L is not a multiple of chunk where required */
    PF_ERR_UNSUPPORTED = 3, /* no kernel instance for this (d_k, d_v, r, chunk, dt) */
    PF_ERR_ALIGN = 4,       /* a base address is not 16-byte aligned */
    PF_ERR_WORKSPACE = 5,   /* workspace is NULL or smaller than pf_delta_fwd_workspace_bytes() */
    PF_ERR_LAUNCH = 6,      /* the HIP runtime refused a launch */
    PF_ERR_SCRATCH_LIMIT = 7 /* pf_delta_fwd_static: the call needs more than pf_delta_fwd_static_limit() bytes */
} pf_status;

typedef enum { PF_F32 = 0, PF_BF16 = 1 } pf_dtype;

/* A hipStream_t, passed as an opaque pointer so that this header needs no HIP header.
 * NULL is the default stream. */
typedef void *pf_stream;

/* Library version: major * 10000 + minor * 100 + patch.  Host only. */
int pf_version(void);

/* Static, never-NULL description of a status code.  Host only. */
const char *pf_status_str(pf_status s);

/* Which kernel family would serve these dimensions.  Host only, no GPU needed.
 *   0  unsupported (pf_delta_fwd would return PF_ERR_UNSUPPORTED)
 *   1  generic path: one workgroup per (b, h), fp32 vector arithmetic, chunk state in LDS; both
 *      dtypes, any d_k, d_v, r; the chunk is halved until its working set fits 160 KiB of LDS next
 *      to the fp32 state (unsupported only when not even one token does); L need not be a
 *      multiple of chunk (the tail is a shorter last chunk)
 *   2  MFMA path (PF_BF16 only): d_k in {64, 128}, d_v any multiple of 16 (the state is split into
 *      tiles of 16 or 32 rows of d_v, so d_v need not equal d_k), and a flow block (see
 *      pf_delta_fwd_block) with block * r in {64, 128, 256}, block in {32, 64, 128}.  Any L: the
 *      L % block tokens left over at the end of every (b, h) are taken by the generic kernel
 *      from the state the whole blocks leave behind (the flows compose, Section 3.1).
 *      With few (b, h) pairs and a long L (the plain scan would use at most a quarter of the
 *      GPU) and d_k = d_v, every head is cut into 4 or more segments that are scanned side by side: a
 *      segment acts on the state as S -> S P + H (Proposition 2.1), P and H of all segments are
 *      computed in parallel, composed per head, and the segments re-run from their true
 *      incoming states.  Same results up to rounding; the workspace grows by a few d x d
 *      matrices per segment.
 */
int pf_delta_fwd_supported(int d_k, int d_v, int r, int chunk, pf_dtype dt);

/* Tokens per flow block actually used for these dimensions.  MFMA path: chunk / 2^j (j = 0 included)
 * among the blocks that have a kernel instance: the one of 64 virtual tokens (block * r) if it holds at
 * least 32 tokens; else the largest of at most 128 virtual tokens; else the largest there is (256
 * virtual tokens).  Small blocks are preferred because the per-block hand-over array grows with the
 * square of the block; below 32 tokens the fixed cost of a block outweighs that.  The flow over a chunk
 * is the composition of the flows over consecutive pieces of it (Section 3.1), so O and S_L are the
 * same function of the inputs either way; only the blocking of the arithmetic, hence its rounding,
 * differs.  On the generic path: the requested chunk, halved until its working set fits LDS.  0 when
 * pf_delta_fwd_supported(...) is 0.  Host only. */
int pf_delta_fwd_block(int d_k, int d_v, int r, int chunk, pf_dtype dt);

/* Bytes of device scratch pf_delta_fwd needs for these dimensions (0 for the generic path, for
 * L shorter than one flow block and for unsupported dimensions).  Host only. */
size_t pf_delta_fwd_workspace_bytes(int B, int H, int L, int d_k, int d_v, int r, int chunk,
                                    pf_dtype dt);

/* Which kernels one pf_delta_fwd (or pf_delta_product_fwd) call with these dimensions enqueues, in
 * launch order: the names of the kernel instantiations as a profiler prints them (template
 * arguments included, parameter lists left out), separated by ';', e.g.
 * "pf::flow_kernel<128, 64, 32, false>;pf::scan_kernel<128, 64, 32, 32, true, false>".  Template
 * arguments: d_k, virtual tokens per block, tokens per block; for the scan kernel then the d_v rows
 * one workgroup owns and whether it reads out O; last, whether the instance is the one for general
 * drivers.  At most cap - 1
 * characters and a terminating NUL are written to buf (buf may be NULL); the return value is the
 * length of the whole description (0 for unsupported or invalid dimensions).  Depends on the
 * compute-unit count of the current device where the d_v tile does (256 when no device answers).
 * Meant for profiles and benchmarks that must name what they measured.  Host only. */
size_t pf_delta_fwd_describe(int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_dtype dt,
                             char *buf, size_t cap);

/*
 * Chunked forward of the rank-r delta rule (problem statement: Sections 1.1, 1.3, 3.1;
 * method: Section 3 steps 1-3 and Theorem 3.2).
 *
 *   Q     [B, H, L, d_k]      dt     in
 *   K     [B, H, L, r, d_k]   dt     in   (r keys per token = L*r "virtual tokens")
 *   V     [B, H, L, r, d_v]   dt     in
 *   beta  [B, H, L, r]        dt     in
 *   S0    [B, H, d_v, d_k]    fp32   in   initial state; NULL means zeros
 *   O     [B, H, L, d_v]      dt     out  o_t = S_t q_t (state AFTER token t)
 *   S_L   [B, H, d_v, d_k]    fp32   out  final state; NULL means "do not write".
 *                                         S_L == S0 (in-place state) is allowed.
 *   workspace / workspace_bytes      device scratch of at least
 *                                    pf_delta_fwd_workspace_bytes(...) bytes (may be NULL when
 *                                    that is 0).  Contents are overwritten.
 *   stream                           hipStream_t the kernels are enqueued on
 *
 * O and S_L must not overlap any input except S_L == S0.
 * Returns PF_OK after enqueueing, else the first failed check (see pf_status).
 * L == 0 is valid: the five sequence pointers may then be NULL, nothing is written to O and
 * S_L receives S0 (or zeros).
 */
pf_status pf_delta_fwd(const void *Q, const void *K, const void *V, const void *beta,
                       const float *S0, void *O, float *S_L,
                       int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_dtype dt,
                       void *workspace, size_t workspace_bytes, pf_stream stream);

/*
 * pf_delta_fwd for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and error behaviour as pf_delta_fwd without the workspace pair; the scratch
 * the kernels need (T and P of every flow block, the per-segment matrices of the segment-parallel
 * scan, the state handed to the tail) lives in a buffer of pf_delta_fwd_static_limit() bytes
 * (32 MiB) inside the library's code object, one copy per GPU, held until the process ends.
 * The call allocates nothing, frees nothing and calls no allocating routine.
 *
 *   - A call whose pf_delta_fwd_workspace_bytes(...) exceeds the limit returns
 *     PF_ERR_SCRATCH_LIMIT and does nothing (d = 128, r = 2, chunk 64 needs 48 KiB per block
 *     of 64 tokens, so about B * H * L = 43 000 token-heads fit; d = 64, r = 1: 16 KiB per block).
 *   - Every call on a GPU shares that GPU's buffer: calls that may overlap in time on one GPU
 *     (different streams, different host threads) race; order them on one stream.  Nothing in
 *     the buffer has to start at zero, so nothing is cleared between calls.
 *   - The buffer's device address is looked up at the first call on each device (or by
 *     pf_init); make that first call, or pf_init(), outside graph capture.
 *
 * pf_init(): optional set-up for the current device (looks up the static buffer, asks the
 * compute-unit count); PF_OK or PF_ERR_LAUNCH.  pf_delta_fwd_static_limit(): host only.
 */
pf_status pf_init(void);
size_t pf_delta_fwd_static_limit(void);
pf_status pf_delta_fwd_static(const void *Q, const void *K, const void *V, const void *beta,
                              const float *S0, void *O, float *S_L,
                              int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_dtype dt,
                              pf_stream stream);

/*
 * Product form of the rank-r transition (the DeltaProduct-style reading that Section 1 cites, as
 * opposed to the additive rank-r increment of Section 3.1 that pf_delta_fwd computes): the r
 * (k, v, beta) triples of a token are applied one after another,
 *
 *     S <- S (I - beta_{t,j} k_{t,j} k_{t,j}^T) + beta_{t,j} v_{t,j} k_{t,j}^T     j = 0 .. r-1,
 *     o_t = S_t q_t   after the r-th,
 *
 * i.e. the rank-1 delta rule of Section 1.3 over the L*r virtual tokens, read out at every r-th.
 * Same chunk flow with one change: the mask M of Theorem 3.2 is strict in the virtual token instead
 * of strict in time (the readout mask is unchanged).  Arguments, workspace size
 * (pf_delta_fwd_workspace_bytes), kernel families (pf_delta_fwd_supported) and error behaviour are
 * those of pf_delta_fwd.  For r = 1 the two entry points compute the same thing.
 */
pf_status pf_delta_product_fwd(const void *Q, const void *K, const void *V, const void *beta,
                               const float *S0, void *O, float *S_L,
                               int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_dtype dt,
                               void *workspace, size_t workspace_bytes, pf_stream stream);

/*
 * Step sizes of the exact rank-1 flow (Section 3.3, product of exponentials): for rank-1 increments
 * exp(a b^T) = Id + ((e^x - 1) / x) a b^T with x = <b, a>; under the delta mapping x = -beta |k|^2, so
 * the exact step over one (k, v, beta) is the delta-rule step with
 *
 *     beta_eff = (1 - exp(-beta |k|^2)) / |k|^2        (beta itself where k = 0)
 *
 * in place of beta, for the transition and for the input term alike (the input increment is
 * carried by the same flow).  Feeding beta_eff to pf_delta_fwd with r = 1, or to pf_delta_product_fwd
 * with any r, replaces the Euler discretisation of Section 3.1 by the exact exponential of every
 * rank-1 increment.
 *
 *   K         [B, H, L, r, d_k]   dt   in
 *   beta      [B, H, L, r]        dt   in
 *   beta_out  [B, H, L, r]        dt   out   may be the same buffer as beta
 *
 * fp32 arithmetic; the result is rounded to dt.  Any d_k.  Error behaviour as for pf_delta_fwd.
 */
pf_status pf_beta_exponential(const void *K, const void *beta, void *beta_out,
                              int B, int H, int L, int d_k, int r, pf_dtype dt, pf_stream stream);

/*
 * The same chunked forward for general low-rank drivers (Section 3.1, before the delta mapping
 * of its Remark): per (b, h), with A_t, B_t in R^{d_k x r} and Atil_t in R^{d_v x r} stored by
 * column,
 *
 *   S_t = S_{t-1} + S_{t-1} A_t B_t^T + Atil_t B_t^T ,     o_t = S_t q_t .
 *
 *   Q     [B, H, L, d_k]      dt     in
 *   A     [B, H, L, r, d_k]   dt     in   column j of A_t is A[b, h, t, j, :]
 *   Atil  [B, H, L, r, d_v]   dt     in
 *   Bm    [B, H, L, r, d_k]   dt     in
 *   S0, O, S_L, stream               as for pf_delta_fwd
 *
 * The delta rule is the special case A = beta k, Atil = -beta v, B = -k.  Served by the generic
 * kernel family only (pf_flow_fwd_supported: 1 unless not even one token's working set fits LDS;
 * the chunk is halved until it fits, as for pf_delta_fwd);
 * needs no workspace; L need not be a multiple of chunk; L == 0 is valid as for pf_delta_fwd.
 * Same error behaviour as pf_delta_fwd.
 */
int pf_flow_fwd_supported(int d_k, int d_v, int r, int chunk, pf_dtype dt);
pf_status pf_flow_fwd(const void *Q, const void *A, const void *Atil, const void *Bm,
                      const float *S0, void *O, float *S_L,
                      int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_dtype dt,
                      pf_stream stream);

/*
 * pf_flow_fwd on the MFMA kernels (PF_BF16 only): the chunk flow of Theorem 3.2 as printed, with
 * the system matrix Id - M (.) A B^T built from two operand arrays (rows from A, columns from B), its
 * inverse T by the same block substitution, P = Mbar (.) Q B^T, and per block
 *
 *   U_eff = T (Atil + A S_c^T),   O_c = Q S_c^T + P U_eff,   S_c+1 = S_c + U_eff^T B .
 *
 * d_k in {64, 128}, d_v a multiple of 16, flow blocks of at most 128 virtual tokens:
 * pf_flow_fwd_mfma_block returns the block used (chosen as for pf_delta_fwd_block, among blocks with
 * block * r <= 128), 0 when none exists (then PF_ERR_UNSUPPORTED: use pf_flow_fwd).  Any L: the
 * L % block tokens at the end of every (b, h) go through the generic kernel.  workspace: at least
 * pf_flow_fwd_mfma_workspace_bytes(...) bytes of device scratch, overwritten.  Arguments otherwise as
 * pf_flow_fwd, errors as pf_delta_fwd.
 */
int pf_flow_fwd_mfma_block(int d_k, int d_v, int r, int chunk, pf_dtype dt);
size_t pf_flow_fwd_mfma_workspace_bytes(int B, int H, int L, int d_k, int d_v, int r, int chunk,
                                        pf_dtype dt);
pf_status pf_flow_fwd_mfma(const void *Q, const void *A, const void *Atil, const void *Bm,
                           const float *S0, void *O, float *S_L,
                           int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_dtype dt,
                           void *workspace, size_t workspace_bytes, pf_stream stream);

/*
 * Step 2 of Section 3 on its own ("parallel compute": the flow of every chunk, no dependence
 * between chunks), MFMA path only: d_k in {64, 128}, d_v a multiple of 16 (the flow does not depend on
 * d_v; the argument is checked so that both split entry points accept the same dimensions) and
 * (chunk * r, chunk) one of (64, 64), (128, 32), (128, 64), (128, 128), (256, 64), (256, 128), else
 * PF_ERR_UNSUPPORTED; L a multiple of chunk, else PF_ERR_SHAPE.  With n = chunk * r and
 * NC = L / chunk, for every (b, h, c):
 *
 *   Cmat = Id + M (.) diag(beta) K K^T,  M[(t,i),(s,j)] = 1 iff s < t     (Theorem 3.2 in delta
 *          variables; Id - M (.) A B^T of the theorem)
 *   T    = Cmat^{-1}                  [n, n]      lower block-triangular; W = T (beta (.) K) and
 *                                                 -U = T (beta (.) V) are W and U of Theorem 3.2
 *   P    = Mbar (.) Q K^T             [chunk, n]  Mbar[t,(s,j)] = 1 iff s <= t (readout mask)
 *
 * Both outputs are bf16, chunk after chunk in (b, h, c) order, each chunk stored as a sequence
 * of 16-row MFMA operand tiles of 64 "lanes" x 8 elements, lane = 16 g + r16.  With MT = n/16,
 * NKT = n/32, CT = chunk/16 and kk(g, e) = 4 g + e (e < 4), 16 + 4 g + e - 4 (e >= 4):
 *
 *   Tt [B,H,NC][MT][NKT][64][8]   T[16 mt + r16][32 kt + kk(g, e)]   written only for 2 kt <= mt
 *   Pt [B,H,NC][CT][NKT][64][8]   P[16 tt + r16][32 kt + kk(g, e)]   written only for
 *                                                                    32 kt < r (16 tt + 16)
 *
 * (tiles outside those ranges are identically zero; they are never read by pf_delta_chunk_scan).
 * Element counts per (b, h): Tt: NC*n*n, Pt: L*n.  Q, K, beta as in pf_delta_fwd.
 */
pf_status pf_delta_chunk_flow(const void *Q, const void *K, const void *beta, void *Tt, void *Pt,
                              int B, int H, int L, int d_k, int d_v, int r, int chunk,
                              pf_stream stream);

/* 1 when pf_delta_chunk_flow and pf_delta_chunk_scan have a kernel instance for these dimensions
 * (the list above), else 0.  Host only. */
int pf_delta_chunk_supported(int d_k, int d_v, int r, int chunk);

/*
 * Step 3 of Section 3 fused with the readout, MFMA path only: hands the state from chunk to
 * chunk and reads out inside each chunk, from the inputs and the arrays pf_delta_chunk_flow wrote:
 *
 *   U_eff = T (beta (.) (V - K S_c^T))   (= U' - W S_c^T: U + W S_0^T of Theorem 3.2, sign folded)
 *   O_c   = Q S_c^T + P U_eff             (discrete flow of Section 3.1 truncated at each token)
 *   S_c+1 = S_c + U_eff^T K               (S_1 of Theorem 3.2)
 *
 * Q, K, V, beta, S0, O, S_L as in pf_delta_fwd (dt = PF_BF16).
 */
pf_status pf_delta_chunk_scan(const void *Q, const void *K, const void *V, const void *beta,
                              const void *Tt, const void *Pt, const float *S0, void *O, float *S_L,
                              int B, int H, int L, int d_k, int d_v, int r, int chunk,
                              pf_stream stream);

/*
 * Steps 2 and 3 of Section 3 in ONE kernel, for callers without scratch memory: the flow of a
 * block (T and P of Theorem 3.2) is built inside the workgroup that scans the block and never
 * leaves the compute unit, so there is no workspace, and device memory sees Q, K, V, beta once
 * and O once as long as the d_v tiles of a (b, h), which share K and Q through one L2, stay in
 * step (measured 1.01-1.03 times the minimal traffic at 2048 to 8192 tokens per head, 1.4 to
 * 1.8 times at 65536 tokens, where the eight tiles of a head drift apart).  The price: every d_v
 * tile of a (b, h) repeats the block's flow for itself, which on MI355X costs more time than
 * the workspace traffic it saves; pf_delta_fwd therefore uses the two kernels of
 * pf_delta_chunk_flow / pf_delta_chunk_scan and is the faster call wherever a workspace can be
 * had.
 *
 * MFMA path only (PF_BF16): d_k = d_v in {64, 128} and (chunk * r, chunk) one of (64, 64),
 * (64, 32), (128, 32), (128, 64), (128, 128) (pf_delta_fwd_fused_supported returns 1), else
 * PF_ERR_UNSUPPORTED.  The chunk is used as given (no halving); L must be a multiple of chunk
 * (PF_ERR_SHAPE otherwise), L == 0 as for pf_delta_fwd.  product = 0 computes pf_delta_fwd,
 * product != 0 pf_delta_product_fwd.  Q, K, V, beta, S0, O, S_L, stream, errors: as there.
 */
int pf_delta_fwd_fused_supported(int d_k, int d_v, int r, int chunk);
pf_status pf_delta_fwd_fused(const void *Q, const void *K, const void *V, const void *beta,
                             const float *S0, void *O, float *S_L,
                             int B, int H, int L, int d_k, int d_v, int r, int chunk, int product,
                             pf_stream stream);

/*
 * Step 2 of Section 3 by the paper's second construction (Theorem 3.4): W and U of every chunk
 * from the grid recursion W(t_m, t_k) swept along its anti-diagonals, whose cells do not depend on
 * each other; no triangular inverse is formed.  Delta variables as everywhere (A = beta k,
 * Atil = -beta v, B = -k); U obeys the same recursion with Atil as the inhomogeneous term
 * (discrete flow of Section 3.1).  Both dtypes; r in {1, 2, 4}; chunk <= 128; d_k and d_v multiples
 * of 16 (else PF_ERR_UNSUPPORTED, see pf_delta_chunk_sigdelta_supported).  L need not be a
 * multiple of chunk: the last chunk of a head is then shorter.
 *
 *   K, V, beta   as in pf_delta_fwd                                              in
 *   W     [B, H, L, r, d_k]   fp32   out  rows (t, j) of W = (Id - M (.) A B^T)^{-1} A of t's chunk
 *   U     [B, H, L, r, d_v]   fp32   out  rows (t, j) of U = (Id - M (.) A B^T)^{-1} Atil
 *   workspace / workspace_bytes      device scratch of at least
 *                                    pf_delta_chunk_sigdelta_workspace_bytes(...) bytes (the
 *                                    (chunk r)^2 fp32 Gram B^T A of every chunk); overwritten.
 *
 * With these, S_1 = S_0 + (U + W S_0^T)^T B (Theorem 3.2).  The arithmetic is fp32 on the vector
 * ALUs (the Gram of bf16 inputs on MFMA); this entry point exists to measure the construction
 * against the blocked substitution behind pf_delta_chunk_flow and is not used by pf_delta_fwd.
 */
int pf_delta_chunk_sigdelta_supported(int d_k, int d_v, int r, int chunk, pf_dtype dt);
size_t pf_delta_chunk_sigdelta_workspace_bytes(int B, int H, int L, int r, int chunk);
pf_status pf_delta_chunk_sigdelta(const void *K, const void *V, const void *beta, float *W, float *U,
                                  int B, int H, int L, int d_k, int d_v, int r, int chunk, pf_dtype dt,
                                  void *workspace, size_t workspace_bytes, pf_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* PF_H */
