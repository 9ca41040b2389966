"""Helpers for the -m gpu tests: move a seeded workload to the device, call the library,
and compare with the fp64 oracle.  (Not collected by pytest.)"""
import numpy as np


def rel_l2(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    num = np.linalg.norm(x - ref)
    return num / den if den > 0 else num


def to_device(w, inp, B=None, H=None):
    """numpy fp32 inputs with head axis N -> torch tensors shaped [B, H, ...] in the workload's dtype."""
    import torch
    B = w.B if B is None else B
    H = w.H if H is None else H
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    dev = torch.device("cuda:0")

    def up(a, dt):
        t = torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        return t.reshape((B, H) + tuple(a.shape[1:])).to(dt).contiguous()

    out = {k: up(inp[k], tdt) for k in ("Q", "K", "V", "beta")}
    out["S0"] = None if inp["S0"] is None else up(inp["S0"], torch.float32)
    return out


def run_gpu(pf, w, dev, chunk=None):
    import torch
    O, SL = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=chunk or w.chunk)
    torch.cuda.synchronize()
    return O.float().cpu().numpy(), SL.cpu().numpy()


def flat_heads(a):
    return a.reshape((-1,) + a.shape[2:])
