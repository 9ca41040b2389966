"""Parity of pf_delta_chunk_sigdelta (anti-diagonal sweep of Theorem 3.4 on the GPU) with the fp64
statements of the paper: W and U of every chunk against Theorem 3.2 (the triangular inverse) and
against the grid recursion of Theorem 3.4 itself, element by element on seeded inputs.  The sweep
is fp32 arithmetic on exact (bf16 or fp32) inputs, so one bar serves both dtypes: rel. L2 <= 1e-4
(the fp32 bar of the forward)."""
import sys

import numpy as np
import pytest

from paper_2504_00492_amd import synth
from gpu_util import rel_l2, to_device

pytestmark = pytest.mark.gpu
TOL = 1e-4


@pytest.fixture(scope="module")
def pf():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_00492_amd import binding
    return binding


def _run(pf, w, inp):
    import torch
    dev = to_device(w, inp)
    dt = pf.PF_BF16 if w.dtype == "bf16" else pf.PF_F32
    assert pf.pf_delta_chunk_sigdelta_supported(w.d_k, w.d_v, w.r, w.chunk, dt) == 1
    need = pf.pf_delta_chunk_sigdelta_workspace_bytes(w.B, w.H, w.L, w.r, w.chunk)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    W = torch.full((w.B, w.H, w.L, w.r, w.d_k), float("nan"), device="cuda:0")
    U = torch.full((w.B, w.H, w.L, w.r, w.d_v), float("nan"), device="cuda:0")
    st = pf.pf_delta_chunk_sigdelta(dev["K"], dev["V"], dev["beta"], W, U, w.B, w.H, w.L, w.d_k, w.d_v, w.r,
                                    w.chunk, dt, ws, need)
    assert st == pf.PF_OK, pf.pf_status_str(st)
    torch.cuda.synchronize()
    return (W.cpu().numpy().reshape(w.heads, w.L * w.r, w.d_k),
            U.cpu().numpy().reshape(w.heads, w.L * w.r, w.d_v))


@pytest.mark.parametrize("kw", [
    dict(dtype="f32", B=1, H=1, L=64, d_k=16, d_v=16, r=1, chunk=16),                    # cfg0's shape
    dict(dtype="f32", B=1, H=2, L=50, d_k=32, d_v=16, r=2, chunk=16),                    # short last chunk, d_k != d_v
    dict(dtype="bf16", B=1, H=2, L=128, d_k=64, d_v=64, r=1, chunk=64),                  # cfg1's chunk
    dict(dtype="bf16", B=2, H=2, L=128, d_k=128, d_v=128, r=2, chunk=64, reflect_frac=0.1),   # cfg2's chunk
    dict(dtype="bf16", B=1, H=2, L=128, d_k=128, d_v=128, r=4, chunk=64),                # cfg3a's chunk
    dict(dtype="bf16", B=1, H=2, L=256, d_k=128, d_v=128, r=2, chunk=128, reflect_frac=0.1),  # cfg4's: two grid columns per lane
    dict(dtype="bf16", B=1, H=1, L=128 + 70, d_k=128, d_v=128, r=4, chunk=128),          # cfg3b's chunk, last chunk of 70 tokens
    dict(dtype="bf16", B=1, H=3, L=40, d_k=48, d_v=16, r=2, chunk=24),                   # Gram without MFMA (d_k % 32 != 0)
    dict(dtype="f32", B=1, H=1, L=7, d_k=16, d_v=16, r=4, chunk=1),                      # one token per chunk: W = A, U = Atil
])
def test_sigdelta_W_U_match_both_theorems(pf, kw):
    from oracle import chunk_flow_ref as cf
    kw = dict(kw)
    dtype = kw.pop("dtype")
    w = synth.Workload("sig", dtype, seed=31, **{"s0_std": 0.0, "reflect_frac": 0.0, **kw})
    print(f"[case] sigdelta dtype={dtype} B={w.B} H={w.H} L={w.L} d=({w.d_k},{w.d_v}) r={w.r} C={w.chunk}", flush=True)
    sys.stdout.flush()
    inp = synth.make_inputs(w)
    Wg, Ug = _run(pf, w, inp)
    assert np.isfinite(Wg).all() and np.isfinite(Ug).all()      # every row of every chunk was written
    worst = 0.0
    for h in range(w.heads):
        for c0 in range(0, w.L, w.chunk):
            sl = slice(c0, min(c0 + w.chunk, w.L))
            rows = slice(sl.start * w.r, sl.stop * w.r)
            A, At, Bm = cf.delta_drivers(inp["K"][h, sl], inp["V"][h, sl], inp["beta"][h, sl])
            Wr, Ur = cf.chunk_flow(A, At, Bm)                    # Theorem 3.2
            eW, eU = rel_l2(Wg[h, rows], Wr), rel_l2(Ug[h, rows], Ur)
            worst = max(worst, eW, eU)
            assert eW <= TOL and eU <= TOL, (h, c0, eW, eU)
            if c0 == 0 and sl.stop - sl.start <= 32:             # the recursion itself (slow in Python)
                assert rel_l2(Wg[h, rows], cf.sig_delta_grid(A, A, Bm)) <= TOL
                assert rel_l2(Ug[h, rows], cf.sig_delta_grid(At, A, Bm)) <= TOL
    print(f"        worst chunk relL2 = {worst:.3e}", flush=True)


def test_sigdelta_flow_reproduces_the_forward(pf, oracle):
    """W, U from the sweep, put through S_1 = S_0 + (U + W S_0^T)^T B (Theorem 3.2) chunk after chunk on
    the host, give the oracle's final state."""
    from oracle import chunk_flow_ref as cf
    w = synth.Workload("sigfwd", "bf16", 1, 2, 256, 64, 64, 2, 64, seed=32, s0_std=0.3, reflect_frac=0.1)
    print("[case] sigdelta -> state of the forward", flush=True)
    inp = synth.make_inputs(w)
    Wg, Ug = _run(pf, w, inp)
    _, SLref = oracle.delta_fwd(inp["Q"], inp["K"], inp["V"], inp["beta"], inp["S0"], want_O=False)
    for h in range(w.heads):
        S = inp["S0"][h].astype(np.float64)
        for c0 in range(0, w.L, w.chunk):
            rows = slice(c0 * w.r, (c0 + w.chunk) * w.r)
            Bm = -inp["K"][h, c0:c0 + w.chunk].astype(np.float64)
            S = cf.chunk_state(S, Wg[h, rows].astype(np.float64), Ug[h, rows].astype(np.float64), Bm)
        assert rel_l2(S, SLref[h]) <= TOL


def test_sigdelta_argument_checks(pf):
    import torch
    z = torch.zeros(16, device="cuda:0")
    assert pf.pf_delta_chunk_sigdelta_supported(128, 128, 3, 64, pf.PF_BF16) == 0
    assert pf.pf_delta_chunk_sigdelta_supported(128, 128, 2, 256, pf.PF_BF16) == 0
    assert pf.pf_delta_chunk_sigdelta_supported(20, 16, 2, 16, pf.PF_F32) == 0
    call = lambda **k: pf.pf_delta_chunk_sigdelta(*[k.get(n, z) for n in ("K", "V", "beta", "W", "U")], 1, 1,
                                                  k.get("L", 16), 16, 16, k.get("r", 1), 16, pf.PF_F32,
                                                  k.get("ws", z), k.get("wb", 1 << 20), 0)
    assert call(r=3) == pf.PF_ERR_UNSUPPORTED
    assert call(W=None) == pf.PF_ERR_NULL
    assert call(wb=8) == pf.PF_ERR_WORKSPACE
    assert call(ws=None) == pf.PF_ERR_WORKSPACE
    assert call(L=-1) == pf.PF_ERR_SHAPE
    assert call(L=0, ws=None) == pf.PF_OK
