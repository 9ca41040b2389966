"""Parity of pf_delta_product_fwd (r sub-updates of a token applied one after another; the contrast
case to the paper's additive rank-r increment) with the fp64 oracle, element by element on seeded
inputs, through the C ABI.  Same bars as the forward: rel. L2 <= 1e-4 (fp32), <= 2e-2 (bf16)."""
import sys

import numpy as np
import pytest

from paper_2504_00492_amd import synth
from gpu_util import rel_l2, to_device, flat_heads, output_stats, state_errors, assert_parity

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def pf():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_00492_amd import binding
    return binding


def _check(pf, oracle, w, expect_family):
    import torch
    dt = pf.PF_BF16 if w.dtype == "bf16" else pf.PF_F32
    fam = pf.pf_delta_fwd_supported(w.d_k, w.d_v, w.r, w.chunk, dt)
    assert fam == expect_family
    print(f"[case] product {w.name} dtype={w.dtype} B={w.B} H={w.H} L={w.L} d=({w.d_k},{w.d_v}) r={w.r} "
          f"C={w.chunk} family={fam}", flush=True)
    sys.stdout.flush()
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    O, SL = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=w.chunk, product=True)
    torch.cuda.synchronize()
    O, SL = O.float().cpu().numpy(), SL.cpu().numpy()
    Oref, SLref = oracle.delta_product_fwd(inp["Q"], inp["K"], inp["V"], inp["beta"], inp["S0"])
    eO, eS = rel_l2(flat_heads(O), Oref), rel_l2(flat_heads(SL), SLref)
    # and it must NOT be the additive form: for r > 1 the result sits several times closer to the
    # product-form oracle than to the additive one (random unit keys in d = 128 are nearly
    # orthogonal, so the two forms are only a few per cent apart there)
    _, SLadd = oracle.delta_fwd(inp["Q"], inp["K"], inp["V"], inp["beta"], inp["S0"], want_O=False)
    gap = rel_l2(flat_heads(SL), SLadd)
    print(f"        relL2(O)={eO:.3e} relL2(S_L)={eS:.3e}  (additive form is {gap:.2e} away)", flush=True)
    assert np.isfinite(O).all() and np.isfinite(SL).all()
    assert_parity(output_stats(flat_heads(O), Oref), state_errors(flat_heads(SL), SLref), w.dtype)
    if w.r > 1:
        assert gap > 5 * eS


@pytest.mark.parametrize("kw", [
    dict(B=1, H=2, L=48, d_k=16, d_v=16, r=2, chunk=16),
    dict(B=2, H=1, L=37, d_k=12, d_v=20, r=3, chunk=8, s0_std=0.5),     # ragged tail, d_k != d_v
    dict(B=1, H=1, L=16, d_k=32, d_v=24, r=4, chunk=1),                 # chunk = 1: the recurrence itself
])
def test_product_generic_fp32(pf, oracle, kw):
    w = synth.Workload("prodgen", "f32", seed=41, **{"s0_std": 0.0, "reflect_frac": 0.0, **kw})
    _check(pf, oracle, w, expect_family=1)


@pytest.mark.parametrize("name,kw", [
    ("cfg2", dict(B=1, H=4, L=512)),                 # r=2 d=128 C=64
    ("cfg3a", dict(B=1, H=2, L=256)),                # r=4 C=64, nonzero S0
    ("cfg3b", dict(B=1, H=2, L=256)),                # r=4 C=128: runs as flow blocks of 64
    ("cfg4", dict(B=1, H=2, L=512)),                 # r=2 C=128, 10 % near-reflections
    ("cfg2", dict(B=1, H=2, L=64 * 3 + 21)),         # ragged: tail through the generic kernel
    ("cfg1", dict(B=1, H=2, L=256)),                 # r=1: same as the additive form
])
def test_product_mfma_path(pf, oracle, name, kw):
    w = synth.WORKLOADS[name].with_(**kw)
    _check(pf, oracle, w, expect_family=2)


def test_product_segment_parallel(pf, oracle):
    """Few heads and a long sequence: the segment-parallel scan, with the product-form flow."""
    w = synth.WORKLOADS["cfg2"].with_(B=1, H=2, L=64 * 64)
    n = w.chunk * w.r
    plain = w.B * w.H * (w.L // w.chunk) * (n * n + w.chunk * n) * 2
    need = pf.pf_delta_fwd_workspace_bytes(w.B, w.H, w.L, w.d_k, w.d_v, w.r, w.chunk, pf.PF_BF16)
    assert need > plain + 3 * w.B * w.H * 4 * w.d_k * w.d_k * 4      # the segment buffers are planned
    _check(pf, oracle, w, expect_family=2)


# ------------------------------------------------------------------ Section 3.3: exact rank-1 steps
@pytest.mark.parametrize("dtype,dk", [("f32", 16), ("f32", 37), ("bf16", 128), ("bf16", 24), ("bf16", 5)])
def test_beta_exponential_matches_closed_form(pf, dtype, dk):
    import torch
    from oracle import chunk_flow_ref as cf
    print(f"[case] beta_exponential dtype={dtype} d_k={dk}", flush=True)
    rng = np.random.default_rng(7)
    B, H, L, r = 2, 3, 50, 2
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    K = torch.from_numpy((rng.standard_normal((B, H, L, r, dk)) * rng.uniform(0.0, 1.5, (B, H, L, r, 1))).astype(np.float32))
    K[0, 0, 3] = 0.0                                             # a zero key: beta passes through
    beta = torch.from_numpy(rng.uniform(0.0, 3.0, (B, H, L, r)).astype(np.float32))
    Kd, bd = K.to("cuda:0").to(tdt).contiguous(), beta.to("cuda:0").to(tdt).contiguous()
    out = torch.full_like(bd, float("nan"))
    dt = pf.PF_F32 if dtype == "f32" else pf.PF_BF16
    assert pf.pf_beta_exponential(Kd, bd, out, B, H, L, dk, r, dt) == pf.PF_OK
    torch.cuda.synchronize()
    ref = cf.exp_rank1_beta(Kd.float().cpu().numpy(), bd.float().cpu().numpy())   # from the values the GPU saw
    got = out.float().cpu().numpy().astype(np.float64)
    bar = 2e-6 if dtype == "f32" else 2.0 ** -8                  # bf16: one rounding of the result
    assert np.all(np.abs(got - ref) <= bar * np.abs(ref) + 1e-30), np.abs(got / np.where(ref == 0, 1, ref) - 1).max()
    assert np.array_equal(got[0, 0, 3], bd.float().cpu().numpy()[0, 0, 3].astype(np.float64))
    # in place
    assert pf.pf_beta_exponential(Kd, bd, bd, B, H, L, dk, r, dt) == pf.PF_OK
    torch.cuda.synchronize()
    assert torch.equal(bd, out)
    assert pf.pf_beta_exponential(None, bd, bd, B, H, L, dk, r, dt) == pf.PF_ERR_NULL
    assert pf.pf_beta_exponential(Kd, bd, bd, B, H, L, dk, 0, dt) == pf.PF_ERR_SHAPE
    assert pf.pf_beta_exponential(Kd, bd, bd, B, H, L, dk, r, 9) == pf.PF_ERR_UNSUPPORTED


def test_exponential_product_flow_end_to_end(pf):
    """pf_beta_exponential followed by pf_delta_product_fwd is the product of exponentials of
    Section 3.3 with its inputs: checked against scipy's expm of every rank-1 increment's augmented
    generator, virtual token by virtual token (fp32 path, small)."""
    import torch
    from scipy.linalg import expm
    print("[case] exponential product flow", flush=True)
    rng = np.random.default_rng(8)
    L, r, dk, dv, C = 24, 2, 16, 16, 8
    K = rng.standard_normal((L, r, dk)) * 0.6
    V = rng.standard_normal((L, r, dv))
    beta = rng.uniform(0.2, 2.5, (L, r))
    Q = rng.standard_normal((L, dk))
    S0 = rng.standard_normal((dv, dk)) * 0.3
    f32 = lambda a: np.asarray(a, dtype=np.float32)
    t = lambda a: torch.from_numpy(f32(a)).to("cuda:0")[None, None].contiguous()
    Kd, Vd, bd, Qd, Sd = t(K), t(V), t(beta), t(Q), t(S0)
    assert pf.pf_beta_exponential(Kd, bd, bd, 1, 1, L, dk, r, pf.PF_F32) == pf.PF_OK
    O, SL = pf.delta_fwd(Qd, Kd, Vd, bd, Sd, chunk=C, product=True)
    torch.cuda.synchronize()
    K, V, beta, Q, S = (f32(a).astype(np.float64) for a in (K, V, beta, Q, S0))
    Oref = np.zeros((L, dv))
    for tt in range(L):
        for j in range(r):
            gen = np.zeros((dk + dv, dk + dv))
            gen[:dk, :dk] = np.outer(beta[tt, j] * K[tt, j], -K[tt, j])            # a b^T
            gen[dk:, :dk] = np.outer(-beta[tt, j] * V[tt, j], -K[tt, j])           # atil b^T
            E = expm(gen)
            S = S @ E[:dk, :dk] + E[dk:, :dk]
        Oref[tt] = S @ Q[tt]
    assert rel_l2(O[0, 0].cpu().numpy(), Oref) <= 1e-4
    assert rel_l2(SL[0, 0].cpu().numpy(), S) <= 1e-4
