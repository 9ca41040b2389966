"""Host-side properties of the dimension queries of include/pf.h over random dimensions (no GPU):
what one query says must agree with what the others say."""
import pytest
from hypothesis import given, settings, strategies as st

from test_abi_host import pf  # noqa: F401  (fixture: builds / loads the library)

DIMS = st.sampled_from([16, 24, 32, 48, 64, 72, 96, 128, 160, 256])
RANK = st.sampled_from([1, 2, 3, 4, 8])
CHUNK = st.sampled_from([1, 8, 16, 32, 48, 64, 128, 256, 512])


@settings(max_examples=300, deadline=None)
@given(dk=DIMS, dv=DIMS, r=RANK, chunk=CHUNK, bf=st.booleans(), B=st.integers(1, 4), H=st.integers(1, 64),
       L=st.integers(0, 5000))
def test_queries_agree(pf, dk, dv, r, chunk, bf, B, H, L):  # noqa: F811
    dt = pf.PF_BF16 if bf else pf.PF_F32
    fam = pf.pf_delta_fwd_supported(dk, dv, r, chunk, dt)
    blk = pf.pf_delta_fwd_block(dk, dv, r, chunk, dt)
    ws = pf.pf_delta_fwd_workspace_bytes(B, H, L, dk, dv, r, chunk, dt)
    names = pf.pf_delta_fwd_describe(B, H, L, dk, dv, r, chunk, dt)
    assert fam in (0, 1, 2)
    assert (blk == 0) == (fam == 0) and (names == []) == (fam == 0)
    if fam == 0:
        assert ws == 0
        return
    assert 1 <= blk <= chunk
    if fam == 2:
        # MFMA path: bf16, d_k with an instance, d_v in 16-row tiles; the block is chunk / 2^j and has an instance
        assert bf and dk in (64, 128) and dv % 16 == 0
        q = chunk // blk
        assert blk * q == chunk and q & (q - 1) == 0
        assert pf.pf_delta_chunk_supported(dk, dv, r, blk) == 1
        assert blk * r in (64, 128, 256)
        if L >= blk:
            n, whole = blk * r, B * H * (L - L % blk)
            assert ws >= whole // blk * n * n * 2 + whole * n * 2 and ws % 256 == 0
            assert names[0].startswith("pf::flow_kernel<%d, %d, %d" % (dk, n, blk))
            assert any(x.startswith("pf::scan_kernel<%d, %d, %d" % (dk, n, blk)) for x in names)
            assert (names[-1].startswith("pf::generic_kernel")) == (L % blk != 0)
        else:
            assert ws == 0 and names == ["pf::generic_kernel<unsigned short, false>"]
    else:
        assert ws == 0 and len(names) == 1 and names[0].startswith("pf::generic_kernel<")
    # the static-scratch entry accepts exactly what fits its buffer
    assert pf.pf_delta_fwd_static_limit() == 32 << 20
    # the one-kernel form: only d_k = d_v, and never for blocks beyond 128 virtual tokens
    if pf.pf_delta_fwd_fused_supported(dk, dv, r, chunk):
        assert dk == dv and dk in (64, 128) and chunk * r in (64, 128)
    # general drivers on the MFMA kernels: blocks of at most 128 virtual tokens
    g = pf.pf_flow_fwd_mfma_block(dk, dv, r, chunk, dt)
    if g:
        assert bf and g * r <= 128 and chunk % g == 0 and dk in (64, 128) and dv % 16 == 0
        assert pf.pf_flow_fwd_mfma_workspace_bytes(B, H, L, dk, dv, r, chunk, dt) >= (0 if L < g else 1)
    else:
        assert pf.pf_flow_fwd_mfma_workspace_bytes(B, H, L, dk, dv, r, chunk, dt) == 0
