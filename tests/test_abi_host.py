"""Host-side checks of the C ABI: the library loads, exports what include/pf.h declares, and
every argument check returns its code before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2504_00492_amd", "libpf.so")


@pytest.fixture(scope="module")
def pf():
    if not os.path.exists(LIB):
        from paper_2504_00492_amd import build
        build.build_library()
    from paper_2504_00492_amd import binding
    return binding


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "pf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pf_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(pf):
    names = _declared_functions()
    assert "pf_delta_fwd" in names and len(names) >= 7
    lib = ctypes.CDLL(LIB)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(pf.EXPORTS) == names


def test_version_and_status_strings(pf):
    assert pf.pf_version() >= 100
    seen = {pf.pf_status_str(s) for s in range(8)}
    assert len(seen) == 8 and all(seen)
    assert pf.pf_status_str(99) == "unknown status"


def test_flow_block(pf):
    F32, BF = pf.PF_F32, pf.PF_BF16
    assert pf.pf_delta_fwd_block(128, 128, 2, 64, BF) == 32             # 64 virtual tokens preferred (>= 32 tokens)
    assert pf.pf_delta_fwd_block(128, 128, 2, 128, BF) == 32            # 256 virtual tokens -> 4 x 64
    assert pf.pf_delta_fwd_block(128, 128, 4, 128, BF) == 32            # r = 4: 64 virtual tokens would be 16 tokens -> 128
    assert pf.pf_delta_fwd_block(128, 128, 4, 64, BF) == 32
    assert pf.pf_delta_fwd_block(128, 128, 1, 128, BF) == 64            # r = 1: blocks of 64 tokens
    assert pf.pf_delta_fwd_block(128, 128, 1, 32, BF) == 0 or pf.pf_delta_fwd_supported(128, 128, 1, 32, BF) == 1   # no 32-token r = 1 instance
    assert pf.pf_delta_fwd_block(128, 128, 8, 64, BF) == 4              # no MFMA instance for r = 8: generic path, 4 tokens
    assert pf.pf_delta_fwd_block(128, 128, 8, 32, BF) == 4              # (256, 32) has no instance, 16 x 8 neither
    assert pf.pf_delta_fwd_block(64, 64, 1, 512, BF) == 64
    assert pf.pf_delta_fwd_block(64, 64, 2, 64, BF) == 32
    assert pf.pf_delta_fwd_block(16, 16, 1, 16, F32) == 16             # generic path: the chunk itself
    # workspace follows the block, not the requested chunk
    assert (pf.pf_delta_fwd_workspace_bytes(2, 16, 8192, 128, 128, 4, 128, BF)
            == pf.pf_delta_fwd_workspace_bytes(2, 16, 8192, 128, 128, 4, 64, BF))
    # the split entry points take every (chunk * r, chunk) that has an instance, and nothing else
    assert pf.pf_delta_chunk_supported(128, 128, 2, 128) == 1 and pf.pf_delta_chunk_supported(128, 128, 4, 64) == 1
    assert pf.pf_delta_chunk_supported(128, 128, 4, 128) == 0 and pf.pf_delta_chunk_supported(128, 72, 1, 64) == 0
    assert pf.pf_delta_chunk_supported(128, 64, 1, 64) == 1 and pf.pf_delta_chunk_supported(96, 96, 1, 64) == 0
    fake = 0x1000
    assert pf.pf_delta_chunk_flow(fake, fake, fake, fake, fake, 1, 1, 256, 128, 128, 4, 128, 0) == pf.PF_ERR_UNSUPPORTED
    assert pf.pf_delta_chunk_flow(fake, fake, fake, fake, fake, 1, 1, 256, 128, 128, 2, 16, 0) == pf.PF_ERR_UNSUPPORTED
    assert pf.pf_delta_chunk_flow(fake, fake, fake, fake, fake, 1, 1, 100, 128, 128, 4, 32, 0) == pf.PF_ERR_SHAPE
    assert pf.pf_delta_chunk_flow(fake, fake, fake, fake, fake, 1, 1, 100, 128, 128, 2, 128, 0) == pf.PF_ERR_SHAPE


def test_describe_names_the_kernels_a_call_launches(pf):
    BF, F32 = pf.PF_BF16, pf.PF_F32
    # (the d_v tile depends on the compute-unit count: 256 is assumed when no device answers)
    assert pf.pf_delta_fwd_describe(4, 16, 4096, 128, 128, 2, 64, BF) == [
        "pf::flow_kernel<128, 64, 32, false>", "pf::scan_kernel<128, 64, 32, 32, true, false>"]
    assert pf.pf_delta_fwd_describe(1, 32, 65536, 128, 128, 2, 128, BF) == [           # chunk 128 -> blocks of 32
        "pf::flow_kernel<128, 64, 32, false>", "pf::scan_kernel<128, 64, 32, 16, true, false>"]
    assert pf.pf_delta_fwd_describe(2, 16, 8192, 128, 128, 4, 64, BF) == [
        "pf::flow_kernel<128, 128, 32, false>", "pf::scan_kernel<128, 128, 32, 16, true, false>"]
    seg = pf.pf_delta_fwd_describe(1, 4, 65536, 128, 128, 2, 64, BF)                    # few heads: segments
    assert seg[0] == "pf::flow_kernel<128, 64, 32, false>" and seg[-1] == "pf::scan_kernel<128, 64, 32, 16, true, false>"
    assert seg.count("pf::scan_kernel<128, 64, 32, 16, false, false>") == 2 and "pf::segment_compose_kernel" in seg
    assert pf.pf_delta_fwd_describe(1, 4, 100, 128, 128, 2, 64, BF)[-1] == "pf::generic_kernel<unsigned short, false>"
    assert pf.pf_delta_fwd_describe(1, 1, 64, 16, 16, 1, 16, F32) == ["pf::generic_kernel<float, false>"]
    assert pf.pf_delta_fwd_describe(1, 1, 64, 256, 256, 1, 16, F32) == []               # unsupported
    assert pf.pf_delta_fwd_describe(0, 1, 64, 16, 16, 1, 16, F32) == []                 # invalid
    # a short buffer gets a truncated, terminated string and the full length comes back
    import ctypes
    from paper_2504_00492_amd.binding import _lib
    buf = ctypes.create_string_buffer(8)
    n = _lib.pf_delta_fwd_describe(4, 16, 4096, 128, 128, 2, 64, BF, buf, 8)
    assert n == len("pf::flow_kernel<128, 64, 32, false>;pf::scan_kernel<128, 64, 32, 32, true, false>") and buf.value == b"pf::flo"


def test_static_entry_host_checks(pf):
    assert pf.pf_delta_fwd_static_limit() == 32 << 20
    fake = 0x1000
    BF = pf.PF_BF16
    args = (fake, fake, fake, fake, None, fake, None)
    assert pf.pf_delta_fwd_static(*args, 4, 16, 4096, 128, 128, 2, 64, BF, 0) == pf.PF_ERR_SCRATCH_LIMIT
    assert pf.pf_delta_fwd_static(None, fake, fake, fake, None, fake, None, 1, 1, 64, 128, 128, 2, 64, BF, 0) == pf.PF_ERR_NULL
    assert pf.pf_delta_fwd_static(*args, 1, 1, 64, 256, 256, 1, 8, pf.PF_F32, 0) == pf.PF_ERR_UNSUPPORTED
    assert pf.pf_delta_fwd_static(*args, 1, 0, 64, 128, 128, 2, 64, BF, 0) == pf.PF_ERR_SHAPE


def test_fused_entry_host_checks(pf):
    assert pf.pf_delta_fwd_fused_supported(128, 128, 2, 64) == 1
    assert pf.pf_delta_fwd_fused_supported(64, 64, 2, 32) == 1
    assert pf.pf_delta_fwd_fused_supported(128, 128, 4, 64) == 0         # 256 virtual tokens
    assert pf.pf_delta_fwd_fused_supported(128, 64, 1, 64) == 0          # d_k != d_v
    assert pf.pf_delta_fwd_fused_supported(128, 128, 0, 64) == 0
    fake = 0x1000
    call = lambda *a: pf.pf_delta_fwd_fused(*a, 0)
    assert call(fake, fake, fake, fake, None, fake, None, 1, 1, 128, 128, 128, 4, 64, 0) == pf.PF_ERR_UNSUPPORTED
    assert call(fake, fake, fake, fake, None, fake, None, 1, 1, 100, 128, 128, 2, 64, 0) == pf.PF_ERR_SHAPE
    assert call(None, fake, fake, fake, None, fake, None, 1, 1, 128, 128, 128, 2, 64, 0) == pf.PF_ERR_NULL
    assert call(fake + 2, fake, fake, fake, None, fake, None, 1, 1, 128, 128, 128, 2, 64, 0) == pf.PF_ERR_ALIGN
    assert call(fake, fake, fake, fake, None, fake, None, 0, 1, 128, 128, 128, 2, 64, 0) == pf.PF_ERR_SHAPE


def test_supported_families(pf):
    BF, F32 = pf.PF_BF16, pf.PF_F32
    assert pf.pf_delta_fwd_supported(16, 16, 1, 16, F32) == 1          # config 0
    assert pf.pf_delta_fwd_supported(64, 64, 1, 64, BF) == 2           # config 1
    assert pf.pf_delta_fwd_supported(128, 128, 2, 64, BF) == 2         # config 2
    assert pf.pf_delta_fwd_supported(128, 128, 4, 64, BF) == 2         # config 3, chunk 64
    assert pf.pf_delta_fwd_supported(128, 128, 2, 128, BF) == 2        # config 4
    assert pf.pf_delta_fwd_supported(128, 128, 4, 128, BF) == 2        # config 3, chunk 128: two blocks of 64
    assert pf.pf_delta_fwd_supported(128, 128, 8, 64, BF) == 1         # r = 8: no MFMA instance, generic path
    assert pf.pf_delta_fwd_supported(128, 128, 2, 64, F32) == 1        # fp32 at that size: generic path on smaller chunks
    assert pf.pf_delta_fwd_block(128, 128, 2, 64, F32) == 16
    assert pf.pf_delta_fwd_block(16, 16, 1, 16, F32) == 16             # fits as requested
    assert pf.pf_delta_fwd_supported(256, 256, 1, 8, F32) == 0         # the fp32 state alone exceeds LDS
    assert pf.pf_delta_fwd_supported(20, 12, 3, 8, BF) == 1            # odd shape -> generic
    assert pf.pf_delta_fwd_supported(128, 64, 2, 64, BF) == 2          # d_v != d_k: MFMA path, d_v tiles of 16 / 32 rows
    assert pf.pf_delta_fwd_supported(64, 48, 1, 64, BF) == 2
    assert pf.pf_delta_fwd_supported(64, 40, 1, 64, BF) == 1           # d_v not a multiple of 16 -> generic
    assert pf.pf_delta_fwd_supported(96, 128, 1, 64, BF) == 1          # d_k without an instance -> generic
    assert pf.pf_delta_fwd_supported(0, 16, 1, 16, F32) == 0
    assert pf.pf_delta_fwd_supported(16, 16, 1, 16, 7) == 0


def test_workspace_bytes(pf):
    BF = pf.PF_BF16
    assert pf.pf_delta_fwd_workspace_bytes(1, 1, 64, 16, 16, 1, 16, pf.PF_F32) == 0
    b = pf.pf_delta_fwd_workspace_bytes(4, 16, 4096, 128, 128, 2, 64, BF)
    tok = 4 * 16 * 4096
    assert b >= tok // 32 * 64 * 64 * 2 + tok * 64 * 2 and b % 256 == 0           # blocks of 32 tokens, n = 64
    # a ragged tail adds the state hand-over buffer to the whole blocks' scratch
    assert pf.pf_delta_fwd_workspace_bytes(4, 16, 4097, 128, 128, 2, 64, BF) == b + 4 * 16 * 128 * 128 * 4
    assert pf.pf_delta_fwd_workspace_bytes(4, 16, 31, 128, 128, 2, 64, BF) == 0       # shorter than one block
    assert pf.pf_delta_fwd_workspace_bytes(0, 16, 4096, 128, 128, 2, 64, BF) == 0


def test_workspace_of_the_segment_parallel_scan(pf):
    """Few heads, long sequence: 3 d x d fp32 matrices per segment plus the two constants."""
    BF = pf.PF_BF16
    d, r, C, L = 128, 2, 32, 65536        # (chunk 64 runs as blocks of 32 tokens as well)
    n = C * r
    plain = lambda heads: heads * (L // C) * (n * n + C * n) * 2
    b4 = pf.pf_delta_fwd_workspace_bytes(1, 4, L, d, d, r, C, BF)         # 32 chains -> 8 segments
    assert b4 == plain(4) + n * d * 2 + d * d * 4 + 3 * 4 * 8 * d * d * 4
    b8 = pf.pf_delta_fwd_workspace_bytes(1, 8, L, d, d, r, C, BF)         # 64 chains -> 4 segments
    assert b8 == plain(8) + n * d * 2 + d * d * 4 + 3 * 8 * 4 * d * d * 4
    b16 = pf.pf_delta_fwd_workspace_bytes(1, 16, L, d, d, r, C, BF)       # 128 chains: plain scan
    assert b16 == plain(16)
    assert pf.pf_delta_fwd_workspace_bytes(1, 4, 512, d, d, r, C, BF) == plain(4) * 512 // L   # too short to cut


def test_argument_checks_return_before_launch(pf):
    """Fake (never dereferenced) addresses: each call must fail its check on the host."""
    A = 0x10000  # 16-byte aligned fake device address
    BF = pf.PF_BF16
    dims = dict(B=1, H=1, L=128, d_k=128, d_v=128, r=2, chunk=64)

    def call(Q=A, K=A, V=A, beta=A, S0=A, O=A, SL=A, ws=A, wb=1 << 40, dt=BF, fn=pf.pf_delta_fwd, **kw):
        d = dict(dims, **kw)
        return fn(Q, K, V, beta, S0, O, SL, d["B"], d["H"], d["L"], d["d_k"], d["d_v"], d["r"],
                  d["chunk"], dt, ws, wb, 0)

    # the product-form entry point shares every check
    prod = pf.pf_delta_product_fwd
    assert call(fn=prod, V=None) == pf.PF_ERR_NULL
    assert call(fn=prod, r=0) == pf.PF_ERR_SHAPE
    assert call(fn=prod, dt=5) == pf.PF_ERR_UNSUPPORTED
    assert call(fn=prod, O=A + 2) == pf.PF_ERR_ALIGN
    assert call(fn=prod, wb=16) == pf.PF_ERR_WORKSPACE

    assert call(Q=None) == pf.PF_ERR_NULL
    assert call(K=None) == pf.PF_ERR_NULL
    assert call(V=None) == pf.PF_ERR_NULL
    assert call(beta=None) == pf.PF_ERR_NULL
    assert call(O=None) == pf.PF_ERR_NULL
    assert call(B=0) == pf.PF_ERR_SHAPE
    assert call(L=-1) == pf.PF_ERR_SHAPE
    assert call(r=0) == pf.PF_ERR_SHAPE
    assert call(chunk=0) == pf.PF_ERR_SHAPE
    assert call(dt=5) == pf.PF_ERR_UNSUPPORTED
    assert call(dt=pf.PF_F32, d_k=256, d_v=256) == pf.PF_ERR_UNSUPPORTED  # fp32 state of 256 x 256 does not fit LDS
    assert call(Q=A + 2) == pf.PF_ERR_ALIGN
    assert call(SL=A + 4) == pf.PF_ERR_ALIGN
    assert call(ws=None) == pf.PF_ERR_WORKSPACE
    assert call(wb=16) == pf.PF_ERR_WORKSPACE
    assert call(ws=A + 8) == pf.PF_ERR_ALIGN

    flow = pf.pf_delta_chunk_flow
    assert flow(A, A, A, None, A, 1, 1, 128, 128, 128, 2, 64, 0) == pf.PF_ERR_NULL
    assert flow(A, A, A, A, None, 1, 1, 128, 128, 128, 2, 64, 0) == pf.PF_ERR_NULL
    assert flow(A, A, A, A, A, 1, 1, 100, 128, 128, 2, 64, 0) == pf.PF_ERR_SHAPE
    assert flow(A, A, A, A, A, 1, 1, 128, 20, 20, 2, 64, 0) == pf.PF_ERR_UNSUPPORTED
    assert flow(A, A, A, A + 2, A, 1, 1, 128, 128, 128, 2, 64, 0) == pf.PF_ERR_ALIGN
    scan = pf.pf_delta_chunk_scan
    assert scan(A, A, A, A, A, A, A, None, A, 1, 1, 128, 128, 128, 2, 64, 0) == pf.PF_ERR_NULL
    assert scan(A, A, A, A, A, A, A, A, A, 1, 1, 128, 128, 72, 2, 64, 0) == pf.PF_ERR_UNSUPPORTED   # d_v not a multiple of 16
    assert scan(A, A, A, A, A, A, A, A, A + 4, 1, 1, 128, 128, 128, 2, 64, 0) == pf.PF_ERR_ALIGN


def test_general_driver_entry_checks(pf):
    A = 0x10000
    F32, BF = pf.PF_F32, pf.PF_BF16
    assert pf.pf_flow_fwd_supported(16, 16, 1, 16, F32) == 1
    assert pf.pf_flow_fwd_supported(20, 12, 3, 8, BF) == 1
    assert pf.pf_flow_fwd_supported(128, 128, 2, 64, BF) == 1          # runs on chunks of 16 tokens
    assert pf.pf_flow_fwd_supported(300, 300, 1, 8, BF) == 0           # the fp32 state alone exceeds LDS
    assert pf.pf_flow_fwd_supported(16, 16, 1, 16, 9) == 0
    call = lambda Q=A, Ad=A, At=A, Bm=A, S0=A, O=A, SL=A, L=40, dk=16, dv=12, r=2, C=8, dt=F32: \
        pf.pf_flow_fwd(Q, Ad, At, Bm, S0, O, SL, 1, 2, L, dk, dv, r, C, dt, 0)
    assert call(Q=None) == pf.PF_ERR_NULL
    assert call(Ad=None) == pf.PF_ERR_NULL
    assert call(At=None) == pf.PF_ERR_NULL
    assert call(Bm=None) == pf.PF_ERR_NULL
    assert call(O=None) == pf.PF_ERR_NULL
    assert call(L=-3) == pf.PF_ERR_SHAPE
    assert call(r=0) == pf.PF_ERR_SHAPE
    assert call(dk=300, dv=300, C=64) == pf.PF_ERR_UNSUPPORTED
    assert call(dt=4) == pf.PF_ERR_UNSUPPORTED
    assert call(Bm=A + 6) == pf.PF_ERR_ALIGN
    assert call(S0=A + 4) == pf.PF_ERR_ALIGN


def test_inputs_are_seeded_and_bf16_exact():
    import numpy as np
    from paper_2504_00492_amd import synth
    w = synth.WORKLOADS["cfg1"].with_(B=1, H=2, L=128)
    a, b = synth.make_inputs(w), synth.make_inputs(w)
    for k in ("Q", "K", "V", "beta"):
        assert np.array_equal(a[k], b[k])
        assert np.array_equal(synth.round_to_bf16(a[k]), a[k])          # already bf16 values
        assert np.array_equal(synth.bf16_bits_to_f32(synth.bf16_bits(a[k])), a[k])
    assert a["S0"] is None
    h1 = synth.head_inputs(w, 1)
    assert np.array_equal(h1[0], a["Q"][1])
    # unit keys up to bf16 rounding; beta in (0, 1)
    assert np.allclose(np.linalg.norm(a["K"], axis=-1), 1.0, atol=2e-2)
    assert a["beta"].min() > 0 and a["beta"].max() < 1
    w4 = synth.WORKLOADS["cfg4"].with_(L=4096)
    q, k, v, beta, s0 = synth.head_inputs(w4, 0)
    frac = np.mean(np.all(beta >= 1.5, axis=-1))
    assert 0.05 < frac < 0.15 and beta.max() <= 2.0
    w3 = synth.WORKLOADS["cfg3a"].with_(L=64)
    assert abs(float(np.std(synth.head_inputs(w3, 0)[4])) - 0.1) < 0.01


def test_sigdelta_entry_checks(pf):
    """pf_delta_chunk_sigdelta: instance table, workspace size and every check that returns before a launch."""
    assert pf.pf_delta_chunk_sigdelta_supported(128, 128, 2, 64, pf.PF_BF16) == 1
    assert pf.pf_delta_chunk_sigdelta_supported(16, 16, 1, 16, pf.PF_F32) == 1
    assert pf.pf_delta_chunk_sigdelta_supported(128, 128, 3, 64, pf.PF_BF16) == 0      # r in {1, 2, 4}
    assert pf.pf_delta_chunk_sigdelta_supported(128, 128, 2, 129, pf.PF_BF16) == 0     # chunk <= 128
    assert pf.pf_delta_chunk_sigdelta_supported(24, 16, 2, 16, pf.PF_F32) == 0         # d multiple of 16
    assert pf.pf_delta_chunk_sigdelta_supported(16, 16, 1, 16, 7) == 0
    # one (chunk r)^2 fp32 Gram per chunk, the short last chunk included
    assert pf.pf_delta_chunk_sigdelta_workspace_bytes(4, 16, 4096, 2, 64) == 64 * 64 * 128 * 128 * 4
    assert pf.pf_delta_chunk_sigdelta_workspace_bytes(1, 2, 50, 2, 16) == 2 * 4 * 32 * 32 * 4
    assert pf.pf_delta_chunk_sigdelta_workspace_bytes(1, 2, 0, 2, 16) == 0
    p = 1 << 20   # fake, aligned, never dereferenced: every call below fails a check first
    call = lambda K=p, W=p, L=64, r=1, ws=p, wb=1 << 30, dt=pf.PF_F32: pf.pf_delta_chunk_sigdelta(
        K, p, p, W, p, 1, 1, L, 16, 16, r, 16, dt, ws, wb, 0)
    assert call(K=None) == pf.PF_ERR_NULL
    assert call(W=None) == pf.PF_ERR_NULL
    assert call(L=-2) == pf.PF_ERR_SHAPE
    assert call(r=3) == pf.PF_ERR_UNSUPPORTED
    assert call(dt=5) == pf.PF_ERR_UNSUPPORTED
    assert call(ws=None) == pf.PF_ERR_WORKSPACE
    assert call(wb=100) == pf.PF_ERR_WORKSPACE
    assert call(K=p + 2) == pf.PF_ERR_ALIGN
    assert call(ws=p + 4) == pf.PF_ERR_ALIGN
    assert call(L=0, K=None, W=None, ws=None, wb=0) == pf.PF_OK


def test_beta_exponential_checks(pf):
    p = 1 << 20
    f = pf.pf_beta_exponential
    assert f(None, p, p, 1, 1, 8, 16, 1, pf.PF_F32, 0) == pf.PF_ERR_NULL
    assert f(p, p, None, 1, 1, 8, 16, 1, pf.PF_F32, 0) == pf.PF_ERR_NULL
    assert f(p, p, p, 0, 1, 8, 16, 1, pf.PF_F32, 0) == pf.PF_ERR_SHAPE
    assert f(p, p, p, 1, 1, 8, 0, 1, pf.PF_F32, 0) == pf.PF_ERR_SHAPE
    assert f(p, p, p, 1, 1, 8, 16, 1, 3, 0) == pf.PF_ERR_UNSUPPORTED
    assert f(p + 2, p, p, 1, 1, 8, 16, 1, pf.PF_BF16, 0) == pf.PF_ERR_ALIGN
    assert f(None, None, None, 1, 1, 0, 16, 1, pf.PF_BF16, 0) == pf.PF_OK     # empty sequence


def test_header_is_plain_c(pf, tmp_path):
    """include/pf.h compiles as C99 with -pedantic -Werror, and a C program linked against libpf.so
    can call the host-only entry points (no C++ types cross the boundary)."""
    import subprocess
    src = tmp_path / "use_pf.c"
    src.write_text(r'''
#include <stdio.h>
#include "pf.h"
int main(void)
{
    pf_dtype dt = PF_BF16;
    pf_stream s = NULL;
    (void)s;
    printf("%d %s %d %d %lu\n", pf_version(), pf_status_str(PF_ERR_ALIGN),
           pf_delta_fwd_supported(128, 128, 2, 64, dt), pf_delta_fwd_block(128, 128, 4, 128, dt),
           (unsigned long)pf_delta_fwd_workspace_bytes(4, 16, 4096, 128, 128, 2, 64, dt));
    /* every check fails before a launch: NULL inputs */
    return pf_delta_fwd(NULL, NULL, NULL, NULL, NULL, NULL, NULL, 1, 1, 64, 128, 128, 2, 64, dt, NULL, 0, NULL) == PF_ERR_NULL ? 0 : 1;
}
''')
    exe = tmp_path / "use_pf"
    libdir = os.path.dirname(LIB)
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-lpf", f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"],
                   check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == pf.pf_version()
    assert out[-3:] == ["2", "32", str(pf.pf_delta_fwd_workspace_bytes(4, 16, 4096, 128, 128, 2, 64, pf.PF_BF16))]
