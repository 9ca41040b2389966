"""Parity of the HIP path (through the C ABI) with the fp64 oracle, element by element, on
seeded inputs.  Bars (gpu_util.BARS): rel. L2 <= 1e-4 for fp32 inputs, <= 2e-2 for bf16 inputs
(fp32 accumulation), on both O and S_L, for every head on its own; plus a bound on every single
token and on the largest single element.  The recurrence has a unique result, so nothing else
is "also correct"."""
import sys

import numpy as np
import pytest

from paper_2504_00492_amd import synth
from gpu_util import rel_l2, to_device, run_gpu, flat_heads, output_stats, state_errors, assert_parity

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def pf():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_00492_amd import binding
    return binding


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _check(pf, oracle, w, expect_family=None, heads=None):
    fam = pf.pf_delta_fwd_supported(w.d_k, w.d_v, w.r, w.chunk, pf.PF_BF16 if w.dtype == "bf16" else pf.PF_F32)
    if expect_family is not None and w.L % w.chunk == 0:
        assert fam == expect_family, (fam, expect_family)
    _say(f"[case] {w.name} dtype={w.dtype} B={w.B} H={w.H} L={w.L} d=({w.d_k},{w.d_v}) r={w.r} C={w.chunk} family={fam}")
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    O, SL = run_gpu(pf, w, dev)
    Oref, SLref = oracle.delta_fwd(inp["Q"], inp["K"], inp["V"], inp["beta"], inp["S0"])
    assert np.isfinite(O).all() and np.isfinite(SL).all()
    assert_parity(output_stats(flat_heads(O), Oref), state_errors(flat_heads(SL), SLref), w.dtype)
    return O, SL, Oref, SLref


# ------------------------------------------------------------------ generic path (fp32 + odd shapes)
def test_config0_fp32(pf, oracle):
    _check(pf, oracle, synth.WORKLOADS["cfg0"], expect_family=1)


@pytest.mark.parametrize("kw", [
    dict(B=2, H=3, L=40, d_k=12, d_v=20, r=2, chunk=8, s0_std=0.5),      # d_k != d_v, several tiles
    dict(B=1, H=2, L=37, d_k=16, d_v=16, r=3, chunk=8, s0_std=0.3),      # ragged tail (37 = 4*8 + 5), r = 3
    dict(B=1, H=1, L=5, d_k=8, d_v=8, r=1, chunk=16),                    # L < chunk
    dict(B=1, H=2, L=16, d_k=32, d_v=24, r=4, chunk=1),                  # chunk = 1 is the recurrence itself
    dict(B=1, H=1, L=64, d_k=64, d_v=64, r=1, chunk=32, reflect_frac=0.3),
])
def test_generic_fp32_shapes(pf, oracle, kw):
    w = synth.Workload("gen", "f32", seed=11, **{"s0_std": 0.0, "reflect_frac": 0.0, **kw})
    _check(pf, oracle, w, expect_family=1)


@pytest.mark.parametrize("dtype,kw", [
    ("f32", dict(B=1, H=2, L=100, d_k=128, d_v=128, r=2, chunk=64, s0_std=0.2)),   # fp32 at d = 128: chunks of 16 tokens
    ("bf16", dict(B=1, H=2, L=70, d_k=128, d_v=128, r=8, chunk=64)),               # r = 8 has no MFMA instance: chunks of 4
    ("f32", dict(B=1, H=1, L=33, d_k=160, d_v=96, r=1, chunk=128, s0_std=0.1)),    # a state of 96 x 160 leaves room for 32 tokens
])
def test_generic_path_on_smaller_chunks(pf, oracle, dtype, kw):
    """A chunk whose working set does not fit LDS is run as smaller chunks (the flows compose)."""
    w = synth.Workload("gensmall", dtype, seed=13, **{"s0_std": 0.0, "reflect_frac": 0.0, **kw})
    blk = pf.pf_delta_fwd_block(w.d_k, w.d_v, w.r, w.chunk, pf.PF_BF16 if dtype == "bf16" else pf.PF_F32)
    assert 0 < blk < w.chunk
    _check(pf, oracle, w, expect_family=1)


def test_generic_bf16_odd_shape(pf, oracle):
    w = synth.Workload("gen16", "bf16", 2, 2, 48, 24, 40, 2, 8, seed=12, s0_std=0.2)
    _check(pf, oracle, w, expect_family=1)


def test_empty_sequence_returns_initial_state(pf):
    import torch
    dev = torch.device("cuda:0")
    S0 = torch.randn(1, 2, 16, 16, device=dev)
    z = lambda *s: torch.zeros(s, device=dev)
    O, SL = pf.delta_fwd(z(1, 2, 0, 16), z(1, 2, 0, 1, 16), z(1, 2, 0, 1, 16), z(1, 2, 0, 1), S0, chunk=16)
    torch.cuda.synchronize()
    assert O.shape == (1, 2, 0, 16) and torch.equal(SL, S0)


# ------------------------------------------------------------------ chunk flow (Theorem 3.2) on its own
@pytest.mark.parametrize("d,r,C", [(64, 1, 64), (128, 2, 64), (128, 4, 64), (128, 2, 128), (128, 1, 128), (64, 4, 64),
                                   (128, 4, 32), (64, 4, 32)])
def test_chunk_flow_matches_theorem(pf, oracle, d, r, C):
    """T and P of every chunk (decoded from their tiled layouts) against the numpy statement of
    Theorem 3.2: T is the inverse of the system matrix, T (beta K) = W and T (beta V) = -U; then the
    scan entry point on those arrays against the oracle."""
    import torch
    from oracle import chunk_flow_ref as cf
    from gpu_util import untile_rows8
    w = synth.Workload("flow", "bf16", 1, 2, 2 * C, d, d, r, C, seed=21, reflect_frac=0.1)
    _say(f"[case] chunk flow d={d} r={r} C={C}")
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    n, NC = C * r, w.L // C
    mk = lambda m: torch.full((1, 2, NC, m), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    Tt, Pt = mk(n * n), mk(C * n)
    st = pf.pf_delta_chunk_flow(dev["Q"], dev["K"], dev["beta"], Tt, Pt, 1, 2, w.L, d, d, r, C)
    assert st == pf.PF_OK
    O = torch.empty(1, 2, w.L, d, dtype=torch.bfloat16, device="cuda:0")
    SL = torch.empty(1, 2, d, d, dtype=torch.float32, device="cuda:0")
    st = pf.pf_delta_chunk_scan(dev["Q"], dev["K"], dev["V"], dev["beta"], Tt, Pt, None, O, SL, 1, 2, w.L, d, d, r, C)
    assert st == pf.PF_OK
    torch.cuda.synchronize()
    Tt, Pt = (t.float().cpu().numpy() for t in (Tt, Pt))
    MT, NKT, CT = n // 16, n // 32, C // 16
    rows = np.arange(n)
    for h in range(2):
        for c in range(NC):
            sl = slice(c * C, (c + 1) * C)
            A, At, Bm = cf.delta_drivers(inp["K"][h, sl], inp["V"][h, sl], inp["beta"][h, sl])
            Wr, Ur = cf.chunk_flow(A, At, Bm)                     # paper's W and U
            Tr = cf.block_tri_inverse(cf.system_matrix(A, Bm), r)
            Kf = inp["K"][h, sl].reshape(n, d).astype(np.float64)
            mask = cf.inclusive_time_mask(C, r)
            Pr = mask * (inp["Q"][h, sl].astype(np.float64) @ Kf.T)
            Tg = untile_rows8(Tt[0, h, c], MT, NKT, relabel=True)
            Pg = untile_rows8(Pt[0, h, c], CT, NKT, relabel=True)
            # T: tiles (mt, kt) with 2 kt <= mt are written, the rest untouched (NaN) and zero in T
            tile_written = (2 * (rows[None, :] // 32) <= rows[:, None] // 16)
            assert np.array_equal(~np.isnan(Tg), tile_written)
            assert np.all(Tr[~tile_written] == 0)
            Tz = np.where(tile_written, Tg, 0.0)
            assert rel_l2(Tz, Tr) < 1e-2
            assert np.all(Tz[np.triu_indices(n, 1)] == 0)         # exactly lower triangular
            assert rel_l2(Tz @ A.reshape(n, d), Wr) < 1e-2        # W of Theorem 3.2
            assert rel_l2(Tz @ At.reshape(n, d), Ur) < 1e-2       # U of Theorem 3.2
            # P: written tiles carry zeros behind the mask; tiles wholly behind it stay untouched (NaN)
            written = ~np.isnan(Pg)
            assert np.all(written[mask == 1])
            assert np.all(Pg[written & (mask == 0)] == 0)
            assert rel_l2(np.where(written, Pg, 0.0), Pr) < 5e-3
    Oref, SLref = oracle.delta_fwd(inp["Q"], inp["K"], inp["V"], inp["beta"], None)
    assert rel_l2(flat_heads(O.float().cpu().numpy()), Oref) < TOL["bf16"]
    assert rel_l2(flat_heads(SL.cpu().numpy()), SLref) < TOL["bf16"]


# ------------------------------------------------------------------ MFMA path, sizes the oracle does in seconds
@pytest.mark.parametrize("name,kw", [
    ("cfg1", dict(B=2, H=4, L=512)),                 # r=1 d=64 C=64, 8 chunks
    ("cfg2", dict(B=1, H=8, L=512)),                 # r=2 d=128 C=64
    ("cfg3a", dict(B=1, H=4, L=256)),                # r=4 C=64, nonzero S0
    ("cfg4", dict(B=1, H=4, L=1024)),                # r=2 C=128, near-reflection betas
    ("cfg2", dict(B=4, H=16, L=128)),                # 64 heads -> 32-row d_v tiles (other scan instance)
])
def test_mfma_path_reduced_sizes(pf, oracle, name, kw):
    w = synth.WORKLOADS[name].with_(**kw)
    _check(pf, oracle, w, expect_family=2)


@pytest.mark.parametrize("d,r,C", [(64, 2, 64), (64, 4, 64), (64, 2, 128), (128, 1, 64), (128, 1, 128), (64, 1, 64)])
def test_mfma_other_instances(pf, oracle, d, r, C):
    w = synth.Workload("inst", "bf16", 1, 3, 3 * C, d, d, r, C, seed=31, s0_std=0.1, reflect_frac=0.05)
    _check(pf, oracle, w, expect_family=2)


@pytest.mark.parametrize("kw", [
    dict(B=1, H=3, L=256, d_k=128, d_v=64, r=2, chunk=64),                 # d_v < d_k
    dict(B=1, H=2, L=192, d_k=64, d_v=128, r=1, chunk=64, s0_std=0.2),     # d_v > d_k, S0 is 128 x 64
    dict(B=1, H=2, L=160, d_k=128, d_v=48, r=4, chunk=32),                 # d_v = 48: three 16-row tiles
    dict(B=4, H=8, L=128, d_k=64, d_v=256, r=2, chunk=64, s0_std=0.1),     # 32 heads x 8 tiles of 32 rows
    dict(B=1, H=2, L=229, d_k=128, d_v=64, r=2, chunk=64, s0_std=0.1),     # ragged tail through the generic kernel
    dict(B=1, H=2, L=256, d_k=128, d_v=32, r=2, chunk=128),                # chunk 128 -> blocks of 32 tokens
    dict(B=1, H=3, L=128, d_k=64, d_v=16, r=1, chunk=64),                  # a single 16-row tile per head
    dict(B=1, H=1, L=96, d_k=128, d_v=512, r=2, chunk=32, s0_std=0.1),     # d_v = 4 d_k: 32 tiles of one head
])
def test_mfma_path_dv_differs_from_dk(pf, oracle, kw):
    """The state is d_v x d_k; only d_k is a compile-time size of the MFMA kernels."""
    w = synth.Workload("dvdk", "bf16", seed=61, **{"s0_std": 0.0, "reflect_frac": 0.05, **kw})
    _check(pf, oracle, w, expect_family=2)


def test_mfma_single_chunk_and_beta_zero(pf, oracle):
    import torch
    w = synth.WORKLOADS["cfg2"].with_(B=1, H=2, L=64, s0_std=0.2)
    _check(pf, oracle, w, expect_family=2)
    # beta = 0: state must come back bit-identical, O = Q S0^T
    inp = synth.make_inputs(w)
    inp["beta"][:] = 0.0
    dev = to_device(w, inp)
    O, SL = run_gpu(pf, w, dev)
    assert np.array_equal(flat_heads(SL), inp["S0"])
    Oref = np.einsum("nld,nvd->nlv", inp["Q"].astype(np.float64), inp["S0"].astype(np.float64))
    assert rel_l2(flat_heads(O), Oref) < 1e-2


def test_mfma_in_place_state_split_sequence_and_determinism(pf, oracle):
    """S_L may alias S0; one call over [0, L) equals two calls chained through the state
    (Proposition 2.1); reruns are bit-identical (no atomics, fixed reduction order)."""
    import torch
    w = synth.WORKLOADS["cfg4"].with_(B=1, H=2, L=512, s0_std=0.1)
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    B, H, L, r, d = 1, 2, w.L, w.r, w.d_k
    need = pf.pf_delta_fwd_workspace_bytes(B, H, L, d, d, r, w.chunk, pf.PF_BF16)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    O1, S1 = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=w.chunk, workspace=ws)
    O2, S2 = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=w.chunk, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2) and torch.equal(S1, S2)
    # two halves, state updated in place
    half = L // 2
    S = dev["S0"].clone()
    Oa = torch.empty(B, H, half, d, dtype=torch.bfloat16, device="cuda:0")
    Ob = torch.empty_like(Oa)
    sl = lambda t, a, b: t[:, :, a:b].contiguous()
    for (a, b, Oh) in ((0, half, Oa), (half, L, Ob)):
        st = pf.pf_delta_fwd(sl(dev["Q"], a, b), sl(dev["K"], a, b), sl(dev["V"], a, b), sl(dev["beta"], a, b),
                             S, Oh, S, B, H, half, d, d, r, w.chunk, pf.PF_BF16, ws, need)
        assert st == pf.PF_OK
    torch.cuda.synchronize()
    assert torch.equal(torch.cat([Oa, Ob], dim=2), O1) and torch.equal(S, S1)


# ---------------------------------------------------------------- one-kernel forward, no workspace
@pytest.mark.parametrize("d,r,C,B,H,nblk,product", [
    (128, 2, 64, 1, 2, 5, 0),        # 16-row d_v tiles
    (128, 2, 64, 4, 16, 3, 0),       # 64 heads: 32-row d_v tiles
    (128, 4, 32, 1, 3, 6, 0),
    (128, 1, 128, 1, 2, 3, 0),
    (128, 1, 64, 1, 2, 4, 0),
    (64, 1, 64, 2, 2, 4, 0),
    (64, 2, 32, 1, 3, 7, 0),
    (64, 2, 64, 1, 2, 3, 0),
    (64, 4, 32, 1, 2, 4, 0),
    (128, 2, 64, 1, 2, 4, 1),        # product form of the rank-r transition
    (64, 4, 32, 1, 2, 4, 1),
])
def test_fused_entry(pf, oracle, d, r, C, B, H, nblk, product):
    """pf_delta_fwd_fused (flow and scan of a block in one kernel) against the oracle, and against
    pf_delta_fwd on the same inputs (same arithmetic up to the blocking of the flow)."""
    import torch
    assert pf.pf_delta_fwd_fused_supported(d, d, r, C) == 1
    w = synth.Workload("fused", "bf16", B, H, nblk * C, d, d, r, C, seed=71, s0_std=0.1, reflect_frac=0.05)
    _say(f"[case] fused d={d} r={r} C={C} B={B} H={H} L={w.L} product={product}")
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    O = torch.full((B, H, w.L, d), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    SL = torch.full((B, H, d, d), float("nan"), dtype=torch.float32, device="cuda:0")
    st = pf.pf_delta_fwd_fused(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], O, SL, B, H, w.L, d, d, r, C, product)
    assert st == pf.PF_OK
    torch.cuda.synchronize()
    ref = oracle.delta_product_fwd if product else oracle.delta_fwd
    Oref, SLref = ref(inp["Q"], inp["K"], inp["V"], inp["beta"], inp["S0"])
    On, Sn = O.float().cpu().numpy(), SL.cpu().numpy()
    assert np.isfinite(On).all() and np.isfinite(Sn).all()
    assert_parity(output_stats(flat_heads(On), Oref), state_errors(flat_heads(Sn), SLref), "bf16")
    O2, S2 = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=C, product=bool(product))
    torch.cuda.synchronize()
    assert rel_l2(On, O2.float().cpu().numpy()) <= 1e-2 and rel_l2(Sn, S2.cpu().numpy()) <= 1e-2


def test_fused_entry_refuses_what_it_cannot_do(pf):
    import torch
    t = torch.zeros(1 << 16, dtype=torch.bfloat16, device="cuda:0")
    f = torch.zeros(1 << 16, dtype=torch.float32, device="cuda:0")
    call = lambda L, d, r, C: pf.pf_delta_fwd_fused(t, t, t, t, None, t, f, 1, 1, L, d, d, r, C, 0)
    assert pf.pf_delta_fwd_fused_supported(128, 128, 4, 64) == 0          # 256 virtual tokens: no instance
    assert pf.pf_delta_fwd_fused_supported(128, 64, 2, 64) == 0
    assert call(128, 128, 4, 64) == pf.PF_ERR_UNSUPPORTED
    assert call(100, 128, 2, 64) == pf.PF_ERR_SHAPE                      # L not a multiple of the chunk
    assert pf.pf_delta_fwd_fused(None, t, t, t, None, t, f, 1, 1, 64, 128, 128, 2, 64, 0) == pf.PF_ERR_NULL
    # L = 0: the state is handed through
    S0 = torch.randn(1, 1, 64, 64, device="cuda:0")
    SL = torch.zeros_like(S0)
    assert pf.pf_delta_fwd_fused(None, None, None, None, S0, None, SL, 1, 1, 0, 64, 64, 1, 64, 0) == pf.PF_OK
    torch.cuda.synchronize()
    assert torch.equal(SL, S0)


# ---------------------------------------------------------------- general drivers (Section 3.1)
@pytest.mark.parametrize("kw", [
    dict(L=48, r=1, dk=16, dv=16, C=16, dtype="f32"),
    dict(L=45, r=2, dk=20, dv=12, C=8, dtype="f32"),      # ragged tail, d_k != d_v
    dict(L=64, r=3, dk=24, dv=40, C=16, dtype="bf16"),
])
def test_general_driver_entry(pf, oracle, kw):
    """pf_flow_fwd against the oracle's general-driver recurrence: drivers that are NOT of delta
    form (A, Atil, B independent), non-symmetric S0, two heads."""
    import torch
    L, r, dk, dv, C = kw["L"], kw["r"], kw["dk"], kw["dv"], kw["C"]
    _say(f"general drivers {kw}")
    rng = np.random.default_rng(77)
    N = 2
    A = (0.3 * rng.standard_normal((N, L, r, dk))).astype(np.float32)
    At = rng.standard_normal((N, L, r, dv)).astype(np.float32)
    Bm = (rng.standard_normal((N, L, r, dk)) / np.sqrt(dk)).astype(np.float32)
    Q = rng.standard_normal((N, L, dk)).astype(np.float32)
    S0 = rng.standard_normal((N, dv, dk)).astype(np.float32)
    tdt = torch.float32 if kw["dtype"] == "f32" else torch.bfloat16
    dev = torch.device("cuda:0")
    up = lambda a: torch.from_numpy(a).to(dev).to(tdt).reshape((1, N) + a.shape[1:]).contiguous()
    tq, ta, tat, tb = up(Q), up(A), up(At), up(Bm)
    ts0 = torch.from_numpy(S0).to(dev).reshape(1, N, dv, dk).contiguous()
    O, SL = pf.flow_fwd(tq, ta, tat, tb, ts0, chunk=C)
    torch.cuda.synchronize()
    O = O.float().cpu().numpy()[0]
    SL = SL.cpu().numpy()[0]
    back = lambda t: t.float().cpu().numpy()[0].astype(np.float64)      # the values the GPU saw
    tol = 1e-4 if kw["dtype"] == "f32" else 2e-2
    for h in range(N):
        Oref, SLref = oracle.flow_head(back(ta)[h], back(tat)[h], back(tb)[h], back(tq)[h], S0[h].astype(np.float64))
        eO, eS = rel_l2(O[h], Oref), rel_l2(SL[h], SLref)
        _say(f"    head {h}: relL2(O)={eO:.3e} relL2(S_L)={eS:.3e}")
        assert eO <= tol and eS <= tol
    # the delta mapping through this entry equals pf_delta_fwd
    K = rng.standard_normal((N, L, r, dk)).astype(np.float32)
    K /= np.linalg.norm(K, axis=-1, keepdims=True)
    V = rng.standard_normal((N, L, r, dv)).astype(np.float32)
    beta = rng.uniform(0, 1, (N, L, r)).astype(np.float32)
    if kw["dtype"] == "f32":
        tk, tv, tbeta = up(K), up(V), up(beta)
        O1, S1 = pf.delta_fwd(tq, tk, tv, tbeta, ts0, chunk=C)
        O2, S2 = pf.flow_fwd(tq, tbeta[..., None] * tk, -(tbeta[..., None] * tv), -tk, ts0, chunk=C)
        torch.cuda.synchronize()
        assert rel_l2(O2.cpu().numpy(), O1.cpu().numpy()) <= 1e-5
        assert rel_l2(S2.cpu().numpy(), S1.cpu().numpy()) <= 1e-5


# ---------------------------------------------------------------- launch-shape edge cases
@pytest.mark.parametrize("kw", [
    dict(N=3, L=256, r=2, dk=128, dv=128, C=64),
    dict(N=2, L=256, r=1, dk=64, dv=64, C=64),
    dict(N=2, L=160, r=4, dk=128, dv=64, C=32),             # d_v != d_k
    dict(N=2, L=229, r=2, dk=64, dv=128, C=128),            # chunk 128 -> blocks of 64; ragged tail (generic kernel)
    dict(N=64, L=128, r=2, dk=128, dv=128, C=64),           # 64 heads: 32-row d_v tiles, single-buffered operands
    dict(N=2, L=192, r=1, dk=128, dv=32, C=128),            # 128 virtual tokens in blocks of 128 tokens
    dict(N=2, L=40, r=2, dk=128, dv=128, C=64),             # shorter than one block: generic kernel alone
])
def test_general_drivers_on_mfma_kernels(pf, oracle, kw):
    """pf_flow_fwd_mfma against the oracle's general-driver recurrence.  Drivers near the delta form
    (so that the state stays bounded over hundreds of tokens) but with A and B independent of each
    other, hence a non-symmetric system matrix; non-zero, non-symmetric S0."""
    import torch
    N, L, r, dk, dv, C = (kw[k] for k in ("N", "L", "r", "dk", "dv", "C"))
    _say(f"[case] general drivers on the MFMA kernels {kw}")
    rng = np.random.default_rng(91)
    unit = lambda x: x / np.linalg.norm(x, axis=-1, keepdims=True)
    k = unit(rng.standard_normal((N, L, r, dk)))
    beta = 1.0 / (1.0 + np.exp(-rng.standard_normal((N, L, r, 1))))
    A = (beta * (k + 0.3 * unit(rng.standard_normal(k.shape)))).astype(np.float32)
    Bm = (-(k + 0.3 * unit(rng.standard_normal(k.shape)))).astype(np.float32)
    At = (rng.standard_normal((N, L, r, dv)) / np.sqrt(dv)).astype(np.float32)
    Q = (rng.standard_normal((N, L, dk)) / np.sqrt(dk)).astype(np.float32)
    S0 = (0.1 * rng.standard_normal((N, dv, dk))).astype(np.float32)
    dev = torch.device("cuda:0")
    up = lambda a: torch.from_numpy(a).to(dev).to(torch.bfloat16).reshape((1, N) + a.shape[1:]).contiguous()
    tq, ta, tat, tb = up(Q), up(A), up(At), up(Bm)
    ts0 = torch.from_numpy(S0).to(dev).reshape(1, N, dv, dk).contiguous()
    blk = pf.pf_flow_fwd_mfma_block(dk, dv, r, C, pf.PF_BF16)
    assert 0 < blk <= C and blk * r <= 128
    need = pf.pf_flow_fwd_mfma_workspace_bytes(1, N, L, dk, dv, r, C, pf.PF_BF16)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    O = torch.full((1, N, L, dv), float("nan"), dtype=torch.bfloat16, device=dev)
    SL = torch.full((1, N, dv, dk), float("nan"), dtype=torch.float32, device=dev)
    st = pf.pf_flow_fwd_mfma(tq, ta, tat, tb, ts0, O, SL, 1, N, L, dk, dv, r, C, pf.PF_BF16, ws, need)
    assert st == pf.PF_OK, pf.pf_status_str(st)
    torch.cuda.synchronize()
    On, Sn = O.float().cpu().numpy()[0], SL.cpu().numpy()[0]
    assert np.isfinite(On).all() and np.isfinite(Sn).all()
    back = lambda t: t.float().cpu().numpy()[0].astype(np.float64)      # the values the GPU saw
    heads = range(N) if N <= 4 else (0, N // 2, N - 1)
    Oref, Sref = [], []
    for h in heads:
        o, sl = oracle.flow_head(back(ta)[h], back(tat)[h], back(tb)[h], back(tq)[h], S0[h].astype(np.float64))
        Oref.append(o)
        Sref.append(sl)
    idx = list(heads)
    assert_parity(output_stats(On[idx], np.stack(Oref)), state_errors(Sn[idx], np.stack(Sref)), "bf16")
    # and the generic kernel (pf_flow_fwd) computes the same thing
    O2, S2 = pf.flow_fwd(tq, ta, tat, tb, ts0, chunk=C)
    torch.cuda.synchronize()
    assert rel_l2(On, O2.float().cpu().numpy()[0]) <= 1e-2 and rel_l2(Sn, S2.cpu().numpy()[0]) <= 1e-2


def test_general_drivers_mfma_argument_checks(pf):
    import torch
    BF = pf.PF_BF16
    assert pf.pf_flow_fwd_mfma_block(128, 128, 2, 64, BF) == 32           # 64 virtual tokens preferred
    assert pf.pf_flow_fwd_mfma_block(128, 128, 2, 128, BF) == 32
    assert pf.pf_flow_fwd_mfma_block(128, 128, 4, 64, BF) == 32
    assert pf.pf_flow_fwd_mfma_block(128, 128, 8, 64, BF) == 0            # r = 8: no instance
    assert pf.pf_flow_fwd_mfma_block(128, 128, 2, 64, pf.PF_F32) == 0
    assert pf.pf_flow_fwd_mfma_block(96, 96, 1, 64, BF) == 0
    t = torch.zeros(1 << 16, dtype=torch.bfloat16, device="cuda:0")
    f = torch.zeros(1 << 16, dtype=torch.float32, device="cuda:0")
    call = lambda *a: pf.pf_flow_fwd_mfma(t, t, t, t, None, t, f, *a)
    assert call(1, 1, 64, 128, 128, 8, 64, BF, t, 1 << 17) == pf.PF_ERR_UNSUPPORTED
    assert call(1, 1, 64, 128, 128, 2, 64, BF, None, 0) == pf.PF_ERR_WORKSPACE
    assert call(1, 1, 64, 128, 128, 2, 64, BF, t, 16) == pf.PF_ERR_WORKSPACE
    assert pf.pf_flow_fwd_mfma(None, t, t, t, None, t, f, 1, 1, 64, 128, 128, 2, 64, BF, t, 1 << 17) == pf.PF_ERR_NULL


def test_more_workgroups_than_the_gpu_holds(pf, oracle):
    """640 heads x 4 d_v tiles = 2560 scan workgroups (ten per CU): workgroups are independent, so
    a grid far beyond what is resident at once must give the same per-head results."""
    w = synth.Workload("many", "bf16", 4, 160, 128, 64, 64, 1, 64, seed=41, s0_std=0.1)
    _say(f"[case] many heads B={w.B} H={w.H} L={w.L} d={w.d_k} r={w.r} C={w.chunk}")
    heads = [0, 1, 255, 256, 511, 639]
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    O, SL = run_gpu(pf, w, dev)
    assert np.isfinite(O).all() and np.isfinite(SL).all()
    sub = {k: (None if inp[k] is None else inp[k][heads]) for k in ("Q", "K", "V", "beta", "S0")}
    Oref, SLref = oracle.delta_fwd(sub["Q"], sub["K"], sub["V"], sub["beta"], sub["S0"])
    for i, h in enumerate(heads):
        eO, eS = rel_l2(flat_heads(O)[h], Oref[i]), rel_l2(flat_heads(SL)[h], SLref[i])
        _say(f"        head {h}: relL2(O)={eO:.3e} relL2(S_L)={eS:.3e}")
        assert eO <= TOL["bf16"] and eS <= TOL["bf16"]


def test_chunk_beyond_one_flow_block(pf, oracle):
    """r = 4, chunk = 128 is 512 virtual tokens: it runs as flow blocks of 32 tokens
    (pf_delta_fwd_block), against the oracle and bit-identical to chunk = 64."""
    import torch
    w = synth.WORKLOADS["cfg3b"].with_(B=1, H=3, L=512)
    assert pf.pf_delta_fwd_block(w.d_k, w.d_v, w.r, w.chunk, pf.PF_BF16) == 32
    _check(pf, oracle, w, expect_family=2)
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    O128, S128 = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=128)
    O64, S64 = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=64)
    torch.cuda.synchronize()
    assert torch.equal(O128, O64) and torch.equal(S128, S64)


@pytest.mark.parametrize("name,kw", [
    ("cfg2", dict(B=1, H=3, L=3 * 64 + 37)),          # whole blocks + a tail of 37 tokens
    ("cfg3b", dict(B=1, H=2, L=2 * 64 + 5)),          # chunk 128 -> blocks of 32, tail 5, S0 != 0
    ("cfg1", dict(B=2, H=2, L=64 + 63)),              # d = 64, tail one token short of a block
    ("cfg4", dict(B=1, H=2, L=100)),                  # chunk 128 -> one block of 64 and a tail of 36
    ("cfg4", dict(B=1, H=2, L=50)),                   # shorter than one block: all of it is tail
])
def test_mfma_path_ragged_length(pf, oracle, name, kw):
    """L need not be a multiple of the flow block: the tail of every head runs on the generic
    kernel from the state the whole blocks leave behind."""
    import torch
    w = synth.WORKLOADS[name].with_(**kw)
    _check(pf, oracle, w, expect_family=None)
    assert pf.pf_delta_fwd_supported(w.d_k, w.d_v, w.r, w.chunk, pf.PF_BF16) == 2
    # S_L == NULL and in-place state with a tail
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    B, H, L, r, d = w.B, w.H, w.L, w.r, w.d_k
    need = pf.pf_delta_fwd_workspace_bytes(B, H, L, d, d, r, w.chunk, pf.PF_BF16)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda:0")
    O1, S1 = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=w.chunk, workspace=ws)
    O2 = torch.empty_like(O1)
    st = pf.pf_delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], O2, None, B, H, L, d, d, r, w.chunk,
                         pf.PF_BF16, ws, need)
    assert st == pf.PF_OK
    S = dev["S0"].clone() if dev["S0"] is not None else torch.zeros(B, H, d, d, dtype=torch.float32, device="cuda:0")
    O3 = torch.empty_like(O1)
    st = pf.pf_delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], S, O3, S, B, H, L, d, d, r, w.chunk,
                         pf.PF_BF16, ws, need)
    assert st == pf.PF_OK
    torch.cuda.synchronize()
    assert torch.equal(O2, O1) and torch.equal(O3, O1) and torch.equal(S, S1)


def test_calls_can_be_captured_in_a_graph(pf):
    """pf_delta_fwd only enqueues kernels on the given stream (no allocation, no memset, no
    synchronisation), so it can be recorded into a HIP graph; every replay, with eager work and
    synchronisations in between, must reproduce the eager result bit for bit."""
    import torch
    w = synth.WORKLOADS["cfg2"].with_(B=1, H=4, L=256, s0_std=0.1)
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    B, H, L, r, d = w.B, w.H, w.L, w.r, w.d_k
    need = pf.pf_delta_fwd_workspace_bytes(B, H, L, d, d, r, w.chunk, pf.PF_BF16)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    O_e, S_e = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=w.chunk, workspace=ws)
    torch.cuda.synchronize()
    O_g = torch.empty_like(O_e)
    S_g = torch.empty_like(S_e)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        st = pf.pf_delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], O_g, S_g, B, H, L, d, d, r,
                             w.chunk, pf.PF_BF16, ws, need, torch.cuda.current_stream())
        assert st == pf.PF_OK
    for rep in range(3):
        O_g.fill_(float("nan"))
        S_g.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O_g, O_e) and torch.equal(S_g, S_e), f"replay {rep}"
        # eager work between replays (also on the same workspace)
        O2, S2 = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=w.chunk, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(O2, O_e)


def test_calls_on_two_streams_with_their_own_workspaces(pf):
    """Calls that share nothing (own inputs, outputs, workspace) may be in flight together on
    different streams; each gives what it gives alone."""
    import torch
    cases = []
    for seed, name, kw in ((1, "cfg2", dict(B=1, H=8, L=1024)), (2, "cfg3a", dict(B=1, H=4, L=512))):
        w = synth.WORKLOADS[name].with_(seed=seed, **kw)
        dev = to_device(w, synth.make_inputs(w))
        need = pf.pf_delta_fwd_workspace_bytes(w.B, w.H, w.L, w.d_k, w.d_v, w.r, w.chunk, pf.PF_BF16)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
        O_ref, S_ref = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=w.chunk, workspace=ws)
        cases.append((w, dev, ws, need, O_ref, S_ref, torch.cuda.Stream()))
    torch.cuda.synchronize()
    outs = []
    for rep in range(4):
        for w, dev, ws, need, O_ref, S_ref, stream in cases:
            O = torch.empty_like(O_ref)
            S = torch.empty_like(S_ref)
            st = pf.pf_delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], O, S, w.B, w.H, w.L, w.d_k, w.d_v,
                                 w.r, w.chunk, pf.PF_BF16, ws, need, stream)
            assert st == pf.PF_OK
            outs.append((O, S, O_ref, S_ref))
    torch.cuda.synchronize()
    for O, S, O_ref, S_ref in outs:
        assert torch.equal(O, O_ref) and torch.equal(S, S_ref)


@pytest.mark.parametrize("name,kw", [
    ("cfg2", dict(B=1, H=2, L=4096)),                 # 16 chains -> 16 segments per head
    ("cfg1", dict(B=1, H=1, L=2048, s0_std=0.2)),     # d = 64, one head, nonzero S0
    ("cfg4", dict(B=1, H=3, L=4096, s0_std=0.1)),     # chunk 128, near-reflection betas
    ("cfg2", dict(B=1, H=8, L=4096, s0_std=0.1)),     # 64 chains -> 4 segments per head
])
def test_segment_parallel_scan(pf, oracle, name, kw):
    """Few heads and a long sequence: the library cuts every head into segments that run as
    chains of their own (affine maps of the state compose, Proposition 2.1).  Same results as
    the oracle, and the state may still be updated in place."""
    import torch
    w = synth.WORKLOADS[name].with_(**kw)
    B, H, L, r, d = w.B, w.H, w.L, w.r, w.d_k
    # the segment buffers show in the workspace size: more than T and P alone
    blk = pf.pf_delta_fwd_block(d, d, r, w.chunk, pf.PF_BF16)
    n = blk * r
    plain = B * H * (L // blk) * (n * n + blk * n) * 2
    need = pf.pf_delta_fwd_workspace_bytes(B, H, L, d, d, r, w.chunk, pf.PF_BF16)
    assert need > plain + 3 * B * H * 4 * d * d * 4
    _check(pf, oracle, w, expect_family=2)
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    O1, S1 = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=w.chunk, workspace=ws)
    S = dev["S0"].clone() if dev["S0"] is not None else torch.zeros(B, H, d, d, dtype=torch.float32, device="cuda:0")
    O2 = torch.empty_like(O1)
    st = pf.pf_delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], S, O2, S, B, H, L, d, d, r, w.chunk,
                         pf.PF_BF16, ws, need)
    assert st == pf.PF_OK
    torch.cuda.synchronize()
    assert torch.equal(O2, O1) and torch.equal(S, S1)
