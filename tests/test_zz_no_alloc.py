"""pf_delta_fwd_static (the entry point that allocates nothing: its scratch is a buffer inside the
library's code object) against pf_delta_fwd on the same inputs, through the C ABI.  Both run the
same kernels, so the results must be bit-identical; the oracle bar is checked as well.  Two
calls in a row share the buffer, the second with a smaller input: what the first call left
behind must not show."""
import numpy as np
import pytest

from paper_2504_00492_amd import synth
from gpu_util import to_device, flat_heads, output_stats, state_errors, assert_parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pf():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_00492_amd import binding
    return binding


def _both(pf, oracle, w):
    import torch
    print(f"[case] static scratch {w.name} B={w.B} H={w.H} L={w.L} d={w.d_k} r={w.r} C={w.chunk}", flush=True)
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    B, H, L, d, r = w.B, w.H, w.L, w.d_k, w.r
    need = pf.pf_delta_fwd_workspace_bytes(B, H, L, d, d, r, w.chunk, pf.PF_BF16)
    assert 0 < need <= pf.pf_delta_fwd_static_limit()
    mk = lambda: (torch.full((B, H, L, d), float("nan"), dtype=torch.bfloat16, device="cuda:0"),
                  torch.full((B, H, d, d), float("nan"), dtype=torch.float32, device="cuda:0"))
    O1, S1 = mk()
    st = pf.pf_delta_fwd_static(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], O1, S1, B, H, L, d, d, r,
                                w.chunk, pf.PF_BF16)
    assert st == pf.PF_OK, pf.pf_status_str(st)
    O2, S2 = mk()
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    st = pf.pf_delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], O2, S2, B, H, L, d, d, r, w.chunk,
                         pf.PF_BF16, ws, need)
    assert st == pf.PF_OK
    torch.cuda.synchronize()
    assert torch.equal(O1, O2) and torch.equal(S1, S2)
    Oref, SLref = oracle.delta_fwd(inp["Q"], inp["K"], inp["V"], inp["beta"], inp["S0"])
    assert_parity(output_stats(flat_heads(O1.float().cpu().numpy()), Oref),
                  state_errors(flat_heads(S1.cpu().numpy()), SLref), "bf16")


def test_static_scratch_two_calls_in_a_row(pf, oracle):
    assert pf.pf_init() == pf.PF_OK
    big = synth.WORKLOADS["cfg2"].with_(B=1, H=8, L=1024, s0_std=0.1)        # 6 MiB of scratch
    small = synth.WORKLOADS["cfg3a"].with_(B=1, H=2, L=229, seed=9)          # smaller, other instance, ragged tail
    _both(pf, oracle, big)
    _both(pf, oracle, small)


def test_static_scratch_segment_parallel_and_small_dims(pf, oracle):
    _both(pf, oracle, synth.WORKLOADS["cfg1"].with_(B=1, H=2, L=4096, s0_std=0.2))   # few heads, long: segments
    _both(pf, oracle, synth.WORKLOADS["cfg1"].with_(B=2, H=3, L=192))


def test_static_scratch_limit_and_checks(pf):
    import torch
    t = torch.zeros(1 << 16, dtype=torch.bfloat16, device="cuda:0")
    f = torch.zeros(1 << 16, dtype=torch.float32, device="cuda:0")
    lim = pf.pf_delta_fwd_static_limit()
    assert lim == 32 << 20
    # cfg2 at full size needs about 200 MB of scratch: refused before anything is launched
    assert pf.pf_delta_fwd_workspace_bytes(4, 16, 4096, 128, 128, 2, 64, pf.PF_BF16) > lim
    assert pf.pf_delta_fwd_static(t, t, t, t, None, t, f, 4, 16, 4096, 128, 128, 2, 64, pf.PF_BF16) == pf.PF_ERR_SCRATCH_LIMIT
    assert pf.pf_delta_fwd_static(None, t, t, t, None, t, f, 1, 1, 64, 128, 128, 2, 64, pf.PF_BF16) == pf.PF_ERR_NULL
    assert pf.pf_delta_fwd_static(t, t, t, t, None, t, f, 1, 1, 64, 256, 256, 1, 8, pf.PF_F32) == pf.PF_ERR_UNSUPPORTED
    # the generic family needs no scratch at all
    w = synth.WORKLOADS["cfg0"]
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    O = torch.empty(1, 1, w.L, 16, device="cuda:0")
    S = torch.empty(1, 1, 16, 16, device="cuda:0")
    assert pf.pf_delta_fwd_static(dev["Q"], dev["K"], dev["V"], dev["beta"], None, O, S, 1, 1, w.L, 16, 16, 1, 16,
                                  pf.PF_F32) == pf.PF_OK
    O2, S2 = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], None, chunk=16)
    torch.cuda.synchronize()
    assert torch.equal(O, O2) and torch.equal(S, S2)


def test_static_scratch_call_inside_a_graph(pf):
    """What the entry point is for: recorded into a HIP graph (no allocation may happen there).
    Every replay, with eager calls on the same static buffer in between, reproduces the eager
    result bit for bit.  (pf_init and one eager call come first: the buffer's address and the
    kernels' LDS opt-ins are looked up outside the capture.)"""
    import torch
    assert pf.pf_init() == pf.PF_OK
    w = synth.WORKLOADS["cfg2"].with_(B=1, H=4, L=256, s0_std=0.1)
    inp = synth.make_inputs(w)
    dev = to_device(w, inp)
    B, H, L, r, d = w.B, w.H, w.L, w.r, w.d_k
    args = lambda O, S: (dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], O, S, B, H, L, d, d, r, w.chunk, pf.PF_BF16)
    O_e = torch.empty(B, H, L, d, dtype=torch.bfloat16, device="cuda:0")
    S_e = torch.empty(B, H, d, d, dtype=torch.float32, device="cuda:0")
    assert pf.pf_delta_fwd_static(*args(O_e, S_e)) == pf.PF_OK
    torch.cuda.synchronize()
    O_g, S_g = torch.empty_like(O_e), torch.empty_like(S_e)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        st = pf.pf_delta_fwd_static(*args(O_g, S_g), torch.cuda.current_stream())
        assert st == pf.PF_OK
    small = synth.WORKLOADS["cfg1"].with_(B=1, H=2, L=128)
    sdev = to_device(small, synth.make_inputs(small))
    for rep in range(3):
        O_g.fill_(float("nan"))
        S_g.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O_g, O_e) and torch.equal(S_g, S_e), f"replay {rep}"
        # an eager call of another shape on the same static buffer between the replays
        Os = torch.empty(1, 2, 128, 64, dtype=torch.bfloat16, device="cuda:0")
        Ss = torch.empty(1, 2, 64, 64, dtype=torch.float32, device="cuda:0")
        assert pf.pf_delta_fwd_static(sdev["Q"], sdev["K"], sdev["V"], sdev["beta"], None, Os, Ss, 1, 2, 128, 64, 64, 1,
                                      64, pf.PF_BF16) == pf.PF_OK
        torch.cuda.synchronize()
