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


# ---- decoding of the tiled operand arrays of pf_delta_chunk_flow (layouts: include/pf.h)
def _lane_grid():
    lane = np.arange(64)
    return lane & 15, lane >> 4          # r16, g


def untile_rows8(t, ntile, nk, relabel=False):
    """[ntile][nk][64][8] -> matrix [16*ntile, 32*nk]; element (lane, e) sits at row 16 i + r16 and
    column 32 k + 8 g + e (or, with relabel, 32 k + 4 g + e for e < 4 and 32 k + 16 + 4 g + e - 4)."""
    t = np.asarray(t).reshape(ntile, nk, 64, 8)
    r16, g = _lane_grid()
    out = np.full((16 * ntile, 32 * nk), np.nan)
    e = np.arange(8)
    for i in range(ntile):
        for k in range(nk):
            if relabel:
                col = 32 * k + np.where(e[None, :] < 4, 4 * g[:, None] + e[None, :], 16 + 4 * g[:, None] + e[None, :] - 4)
            else:
                col = 32 * k + 8 * g[:, None] + e[None, :]
            out[(16 * i + r16)[:, None], col] = t[i, k]
    return out


def untile_acc4(t, mt, dt):
    """[mt][dt][64][4] -> matrix [16*mt, 16*dt]; element (lane, e) at row 16 i + 4 g + e, column 16 j + r16."""
    t = np.asarray(t).reshape(mt, dt, 64, 4)
    r16, g = _lane_grid()
    out = np.full((16 * mt, 16 * dt), np.nan)
    e = np.arange(4)
    for i in range(mt):
        for j in range(dt):
            out[16 * i + 4 * g[:, None] + e[None, :], (16 * j + r16)[:, None]] = t[i, j]
    return out
