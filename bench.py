#!/usr/bin/env python3
"""Benchmark of the chunked rank-r delta-rule forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4] [--only]

One "step" is one pass of the whole hot path (chunk flow + state scan with fused readout, i.e.
one pf_delta_fwd call) over one batch of seeded synthetic input that is already resident in
HBM.  Prints ONE JSON line.  The headline fields are those of --workload (default: cfg4, the
largest configuration: 32 heads of 65536 tokens, d = 128, r = 2, chunk 128); unless --only is
given, "configs" holds the same measurements for every other configuration (cfg0, cfg1, cfg2,
cfg3a, cfg3b), each with its own K timed steps.  Per workload:
  * "ms_per_step" / "value": K steps timed after W warm-up steps and a settling period of
    further untimed steps (>= 0.15 s of GPU work; the clocks of this GPU need that long), and
    "ms_per_step_first_pass": the K steps timed right after the W warm-up steps, before settling;
  * "kernels": each kernel's average duration, HIP events on the launch stream over K launches
    through the split entry points (same kernels, same arguments, same input rotation), with its
    algorithmic bytes and FLOPs against the HBM and bf16 MFMA peaks;
  * "roofline": the dominant kernel against the roofline that bounds it.  Both kernels sit on the
    HBM side of the ridge (arithmetic intensity about 50-120 flop/B against 2500 TFLOP/s /
    8 TB/s = 312 flop/B), so it is algorithmic bytes (the q, k, v, beta it must read and the o
    it must write) per second against the 8 TB/s HBM peak.  "traffic" is the HBM bytes per launch
    that rocprofv3's counters saw for that kernel (profiles/hbm_traffic.json), taken over only if
    the profiled kernel instantiation is the one this run launched (pf_delta_fwd_describe);
  * "requested_chunk": where pf_delta_fwd runs flow blocks shorter than the requested chunk, the
    two kernels timed at the requested chunk itself through the split entry points (null when no
    instance of that size exists);
  * "fused_kernel": the one-kernel forward (pf_delta_fwd_fused) on the same blocks;
  * "general_drivers": the same forward through the general-driver kernels (pf_flow_fwd_mfma) on
    drivers of the same shape (A = -K / 2, Atil = V, B = K: two operand arrays instead of one).
"cpu_baseline": the fp64 oracle (oracle/, untuned) timed on this machine's host cores on a stated
sample of the headline workload, with the parity of the GPU result on that sample.
Only one GPU is used; --gpus N with N > 1 exits with a message.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_F32_VALU_TFLOPS = 157.3   # MI355X fp32 vector, published (256 CUs x 128 lanes x 2 flop x 2.4 GHz)
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
SETTLE_S = 0.15                # untimed busy time before the settled timed region
LLC_BYTES = 256 * 2 ** 20      # last-level cache: smaller inputs are rotated over several copies
ALL_WORKLOADS = ["cfg0", "cfg1", "cfg2", "cfg3a", "cfg3b", "cfg4"]


def flops_per_token_head(d, r, C):
    """Headline yardstick: algorithmic (masked, useful) FLOPs per token-head of the chunked
    algorithm with flow blocks of C tokens: Gram d r^2 (C-1), forward substitution for W and U
    2 d r^2 (C-1), the three state products (4r+2) d^2, masked Q K^T and P U_eff d r (C+1) each."""
    return 3 * d * r * r * (C - 1) + (4 * r + 2) * d * d + 2 * d * r * (C + 1)


def dense_flops_per_token_head(d, r, C):
    """What full-tile execution would run (no use of the triangular / causal structure):
    6 C r^2 d + (4r+2) d^2 + 4 C r d.  Reported beside the headline, never as the headline."""
    return 6 * C * r * r * d + (4 * r + 2) * d * d + 4 * C * r * d


def kernel_flops_per_token_head(d, r, C):
    """Useful FLOPs each kernel executes per token-head (the explicit inverse of the n x n
    triangular system, about C^2 r^3 / 3, is not counted).
    flow: Gram d r^2 (C-1) + masked Q K^T d r (C+1)
    scan: K S^T, U_eff^T K, Q S^T = (4r+2) d^2; T R = d r^2 C; P U_eff = d r (C+1)."""
    flow = d * r * r * (C - 1) + d * r * (C + 1)
    scan = (4 * r + 2) * d * d + d * r * r * C + d * r * (C + 1)
    return flow, scan


def min_bytes_per_token_head(d, r, e):
    """Read q, r k, r v, r beta; write o."""
    return e * d * (2 + 2 * r) + e * r


def kernel_bytes_per_token_head(d, r, e):
    """Algorithmic bytes per token-head of each kernel: the part of q, k, v, beta, o it cannot
    avoid touching.  The T / P hand-over between the two kernels is not algorithmic; it shows
    up in the measured traffic."""
    flow = e * d * (1 + r) + e * r                # q, k, beta
    scan = e * d * (2 + 2 * r) + e * r            # q, k, v, beta, o
    return flow, scan


def device_inputs(synth, w, dev, torch):
    """Generated head by head on the host (threads: the draws of a head depend on (seed, head)
    alone), uploaded once; resident in HBM before anything is timed."""
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    N, L, r, dk, dv = w.heads, w.L, w.r, w.d_k, w.d_v
    Q = torch.empty((N, L, dk), dtype=tdt, device=dev)
    K = torch.empty((N, L, r, dk), dtype=tdt, device=dev)
    V = torch.empty((N, L, r, dv), dtype=tdt, device=dev)
    beta = torch.empty((N, L, r), dtype=tdt, device=dev)
    S0 = torch.empty((N, dv, dk), dtype=torch.float32, device=dev) if w.s0_std > 0 else None
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        for h, (q, k, v, b, s0) in enumerate(pool.map(lambda i: synth.head_inputs(w, i), range(N))):
            Q[h] = torch.from_numpy(q).to(dev).to(tdt)
            K[h] = torch.from_numpy(k).to(dev).to(tdt)
            V[h] = torch.from_numpy(v).to(dev).to(tdt)
            beta[h] = torch.from_numpy(b).to(dev).to(tdt)
            if S0 is not None:
                S0[h] = torch.from_numpy(s0).to(dev)
    shp = lambda t: t.reshape((w.B, w.H) + tuple(t.shape[1:]))
    return shp(Q), shp(K), shp(V), shp(beta), None if S0 is None else shp(S0)


def time_split(pf, torch, sets, S0, O, SL, dims, block, nwarm, steps, stream):
    """Average duration of the flow and the scan kernel at flow blocks of `block` tokens: HIP events
    on the launch stream around each launch through the split entry points, inputs rotated as in
    the headline loop.  Returns (flow ms, scan ms)."""
    B, H, L, dk, dv, r = dims
    n, NC = block * r, L // block
    dev = O.device
    Tt = torch.empty((B, H, NC, n * n), dtype=torch.bfloat16, device=dev)
    Pt = torch.empty((B, H, NC, block * n), dtype=torch.bfloat16, device=dev)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    for i in range(nwarm + steps):
        q, k, v, b = sets[i % len(sets)]
        j = i - nwarm
        if j >= 0:
            ev[j][0].record(stream)
        st = pf.pf_delta_chunk_flow(q, k, b, Tt, Pt, B, H, L, dk, dv, r, block, stream)
        assert st == pf.PF_OK, st
        if j >= 0:
            ev[j][1].record(stream)
        st = pf.pf_delta_chunk_scan(q, k, v, b, Tt, Pt, S0, O, SL, B, H, L, dk, dv, r, block, stream)
        assert st == pf.PF_OK, st
        if j >= 0:
            ev[j][2].record(stream)
    torch.cuda.synchronize()
    t_flow = sum(a.elapsed_time(b) for a, b, _ in ev) / steps
    t_scan = sum(b.elapsed_time(c) for _, b, c in ev) / steps
    del Tt, Pt
    return t_flow, t_scan


def run_workload(pf, torch, w, inputs, args, traffic_table):
    """All measurements of one workload; returns (result dict, O, SL of input set 0)."""
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    dt = pf.PF_BF16 if w.dtype == "bf16" else pf.PF_F32
    B, H, L, r, dk, dv, C = w.B, w.H, w.L, w.r, w.d_k, w.d_v, w.chunk
    fam = pf.pf_delta_fwd_supported(dk, dv, r, C, dt)
    if fam == 0:
        raise SystemExit(f"bench.py: no kernel instance for workload {w.name}")
    Q, K, V, beta, S0 = inputs
    O = torch.empty((B, H, L, dv), dtype=tdt, device=dev)
    SL = torch.empty((B, H, dv, dk), dtype=torch.float32, device=dev)
    need = pf.pf_delta_fwd_workspace_bytes(B, H, L, dk, dv, r, C, dt)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    # A small workload would sit in the last-level cache if every step read the same buffers:
    # rotate over enough copies of the inputs that each step finds its inputs cold.
    in_bytes = sum(t.numel() * t.element_size() for t in (Q, K, V, beta))
    nsets = 1 if in_bytes >= LLC_BYTES else min(64, -(-(600 * 2 ** 20) // in_bytes))
    sets = [(Q, K, V, beta)] + [tuple(t.clone() for t in (Q, K, V, beta)) for _ in range(nsets - 1)]

    def step(i=0):
        q, k, v, b = sets[i % nsets]
        st = pf.pf_delta_fwd(q, k, v, b, S0, O, SL, B, H, L, dk, dv, r, C, dt, ws, need, stream)
        if st != pf.PF_OK:
            raise pf.PfError(st, "pf_delta_fwd")

    def timed(first):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(first + i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    for i in range(args.warmup):
        step(i)
    ms_first = timed(args.warmup)              # K steps right after the W warm-up steps
    # Keep the GPU busy (untimed) for SETTLE_S seconds, then time K steps again: the first few
    # milliseconds of a burst of launches run up to 20 % slower than the steady state.
    settle_steps = 0
    ts = time.perf_counter()
    while time.perf_counter() - ts < SETTLE_S and settle_steps < 20000:
        for i in range(20):
            step(settle_steps + i)
        settle_steps += 20
        torch.cuda.synchronize()
    ms_per_step = timed(args.warmup)
    step(0)                                    # leave the outputs of input set 0 behind (parity check)
    torch.cuda.synchronize()

    tokens, token_heads = B * L, B * H * L
    block = pf.pf_delta_fwd_block(dk, dv, r, C, dt)
    launched = pf.pf_delta_fwd_describe(B, H, L, dk, dv, r, C, dt)
    f_alg = flops_per_token_head(dk, r, block)
    e = 2 if w.dtype == "bf16" else 4
    min_bytes = min_bytes_per_token_head(dk, r, e) * token_heads
    alg_tflops = f_alg * token_heads / (ms_per_step * 1e-3) / 1e12

    kernels, requested, fused, general = {}, None, None, None
    if fam == 2:
        dims = (B, H, L, dk, dv, r)
        nwarm = min(args.warmup + settle_steps, 200)

        def kinfo(ms, fl, by, name):
            tf = fl * token_heads / (ms * 1e-3) / 1e12
            gb = by * token_heads / (ms * 1e-3) / 1e9
            return {"name": name, "ms": ms, "alg_tflops": tf, "frac_bf16_mfma_peak": tf / PEAK_BF16_TFLOPS,
                    "alg_gbs": gb, "frac_hbm_peak": gb / PEAK_HBM_GBS,
                    "alg_bytes_per_launch": by * token_heads, "flop_per_alg_byte": fl / by}

        name_of = lambda key: next((k for k in launched if k.startswith("pf::" + key)), None)
        t_flow, t_scan = time_split(pf, torch, sets, S0, O, SL, dims, block, nwarm, args.steps, stream)
        f_flow, f_scan = kernel_flops_per_token_head(dk, r, block)
        b_flow, b_scan = kernel_bytes_per_token_head(dk, r, e)
        kernels = {"flow_kernel": kinfo(t_flow, f_flow, b_flow, name_of("flow_kernel")),
                   "scan_kernel": kinfo(t_scan, f_scan, b_scan, name_of("scan_kernel"))}
        dom = "flow_kernel" if t_flow >= t_scan else "scan_kernel"
        roofline = {"bound": "hbm", "kernel": dom, "kernel_name": kernels[dom]["name"],
                    "achieved": kernels[dom]["alg_gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": kernels[dom]["frac_hbm_peak"], "avg_kernel_ms": kernels[dom]["ms"], "traffic": None}
        # counters of a profiled run count only if that run launched this very instantiation
        for key, info in kernels.items():
            rec = traffic_table.get(w.name, {}).get(key)
            info["traffic"] = rec["bytes"] if isinstance(rec, dict) and rec.get("name") == info["name"] else None
        roofline["traffic"] = kernels[dom]["traffic"]
        if kernels["flow_kernel"]["traffic"] and kernels["scan_kernel"]["traffic"]:
            roofline["traffic_both_kernels_over_min_bytes"] = (
                (kernels["flow_kernel"]["traffic"] + kernels["scan_kernel"]["traffic"]) / min_bytes)

        # the two kernels at the requested chunk itself, where the library runs shorter blocks
        if block != C:
            if pf.pf_delta_chunk_supported(dk, dv, r, C) and L % C == 0:
                tf_, ts_ = time_split(pf, torch, sets, S0, O, SL, dims, C, 20, max(10, args.steps // 4), stream)
                requested = {"chunk": C, "virtual_tokens": C * r, "flow_ms": tf_, "scan_ms": ts_,
                             "ms_both": tf_ + ts_, "policy_block": block, "policy_ms_both": t_flow + t_scan}
            else:
                requested = {"chunk": C, "virtual_tokens": C * r, "ms_both": None, "policy_block": block,
                             "why": "no kernel instance for blocks of this many virtual tokens"}
        # (the one-kernel forward is at its best on blocks of 128 virtual tokens)
        fblock = next((c for c in (128 // r, block) if c <= C and C % c == 0 and L % c == 0 and
                       pf.pf_delta_fwd_fused_supported(dk, dv, r, c)), 0)
        if fblock:
            nrep = max(10, args.steps // 4)
            evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(nrep)]
            for i in range(10 + nrep):
                q, k, v, b = sets[i % nsets]
                if i >= 10:
                    evs[i - 10][0].record(stream)
                st = pf.pf_delta_fwd_fused(q, k, v, b, S0, O, SL, B, H, L, dk, dv, r, fblock, 0, stream)
                assert st == pf.PF_OK, st
                if i >= 10:
                    evs[i - 10][1].record(stream)
            torch.cuda.synchronize()
            t_fused = sum(a.elapsed_time(b) for a, b in evs) / nrep
            fused = {"ms": t_fused, "block": fblock, "min_hbm_gbs": min_bytes / (t_fused * 1e-3) / 1e9,
                     "frac_hbm_peak": min_bytes / (t_fused * 1e-3) / 1e9 / PEAK_HBM_GBS}
            step(0)
            torch.cuda.synchronize()
        gblock = pf.pf_flow_fwd_mfma_block(dk, dv, r, C, dt)
        if gblock:
            gneed = pf.pf_flow_fwd_mfma_workspace_bytes(B, H, L, dk, dv, r, C, dt)
            gws = torch.empty(max(gneed, 16), dtype=torch.uint8, device=dev)
            Ag = (K * -0.5).contiguous()
            nrep = max(10, args.steps // 4)
            evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(nrep)]
            for i in range(5 + nrep):
                if i >= 5:
                    evs[i - 5][0].record(stream)
                st = pf.pf_flow_fwd_mfma(Q, Ag, V, K, S0, O, SL, B, H, L, dk, dv, r, C, dt, gws, gneed, stream)
                assert st == pf.PF_OK, st
                if i >= 5:
                    evs[i - 5][1].record(stream)
            torch.cuda.synchronize()
            general = {"ms": sum(a.elapsed_time(b) for a, b in evs) / nrep, "block": gblock}
            del gws, Ag
            step(0)
            torch.cuda.synchronize()
    else:
        tfl = f_alg * token_heads / (ms_per_step * 1e-3) / 1e12
        roofline = {"bound": "alu", "kernel": "generic_kernel", "kernel_name": launched[0] if launched else None,
                    "achieved": tfl, "peak": PEAK_F32_VALU_TFLOPS, "unit": "TFLOP/s",
                    "frac": tfl / PEAK_F32_VALU_TFLOPS, "avg_kernel_ms": ms_per_step, "traffic": None}

    res = {
        "value": tokens / (ms_per_step * 1e-3), "unit": "tokens/s",
        "ms_per_step": ms_per_step, "ms_per_step_first_pass": ms_first,
        "settle_steps": settle_steps,   # untimed steps between the first pass and the settled pass
        "dtype": w.dtype,
        "config": {"workload": f"{w.name}: B={B} H={H} L={L} d_k=d_v={dk} r={r} chunk={C} {w.dtype}",
                   "kernel_family": {1: "generic", 2: "mfma"}[fam], "flow_block": block, "launches": launched},
        "alg_tflops": alg_tflops, "frac_bf16_mfma_peak": alg_tflops / PEAK_BF16_TFLOPS,
        # the same time priced with the full-tile flop count of the blocking that ran (padding and
        # masked-out products included): an upper bound on what the MFMA pipe executed, not a headline
        "dense_tflops": dense_flops_per_token_head(dk, r, block) * token_heads / (ms_per_step * 1e-3) / 1e12,
        "token_heads_per_s": token_heads / (ms_per_step * 1e-3),
        "min_hbm_gbs": min_bytes / (ms_per_step * 1e-3) / 1e9,
        "frac_hbm_peak_min_traffic": min_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "kernels": kernels, "roofline": roofline, "requested_chunk": requested, "fused_kernel": fused,
        "general_drivers": general,
        # inputs + outputs + workspace of one step; when that is below the last-level cache the
        # inputs are rotated over several copies so that each step reads them from HBM
        "working_set_bytes": int(min_bytes + need + B * H * dv * dk * 4),
        "input_sets_rotated": nsets,
    }
    del sets, ws
    return res, O, SL


def compare_solvers(pf, torch, w, inputs, block, flow_ms, steps):
    """Step 2 of Section 3 by the anti-diagonal sweep of Theorem 3.4 next to the blocked substitution."""
    dt = pf.PF_BF16 if w.dtype == "bf16" else pf.PF_F32
    B, H, L, r, dk, dv = w.B, w.H, w.L, w.r, w.d_k, w.d_v
    if not pf.pf_delta_chunk_sigdelta_supported(dk, dv, r, block, dt):
        return None
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    _, K, V, beta, _ = inputs
    sneed = pf.pf_delta_chunk_sigdelta_workspace_bytes(B, H, L, r, block)
    sws = torch.empty(sneed, dtype=torch.uint8, device=dev)
    Wo = torch.empty((B, H, L, r, dk), dtype=torch.float32, device=dev)
    Uo = torch.empty((B, H, L, r, dv), dtype=torch.float32, device=dev)
    nrep = min(10, max(3, steps // 4))
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(nrep)]
    for i in range(1 + nrep):
        if i >= 1:
            evs[i - 1][0].record(stream)
        st = pf.pf_delta_chunk_sigdelta(K, V, beta, Wo, Uo, B, H, L, dk, dv, r, block, dt, sws, sneed, stream)
        assert st == pf.PF_OK, st
        if i >= 1:
            evs[i - 1][1].record(stream)
    torch.cuda.synchronize()
    t_sig = sum(a.elapsed_time(b) for a, b in evs) / nrep
    # useful fp32 operations of the sweep: C(C-1)/2 grid cells, r rows of d_k + d_v columns, 2 + r
    # additions / multiply-adds each (counted as 2 flops), per chunk-head
    sig_flops = (block * (block - 1) // 2) * r * (dk + dv) * (2 + r) * 2 * (B * H * L / block)
    return {
        "sigdelta": {"ms": t_sig, "chunk": block, "n": block * r, "gives": "W, U fp32 (Gram kernel + sweep kernel)",
                     "sweep_tflops_fp32": sig_flops / (t_sig * 1e-3) / 1e12,
                     "frac_fp32_valu_peak": sig_flops / (t_sig * 1e-3) / 1e12 / PEAK_F32_VALU_TFLOPS},
        "block_substitution": {"ms": flow_ms, "chunk": block, "n": block * r,
                               "gives": "T = (Id + G)^-1 and P, bf16 (W = T beta K and U are formed by "
                                        "the scan kernel)"},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="cfg4", help="headline workload: " + ", ".join(ALL_WORKLOADS) +
                    " (see paper_2504_00492_amd/synth.py)")
    ap.add_argument("--only", action="store_true", help="measure the headline workload alone (no 'configs' array)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seq-len", type=int, default=0, help="override the workload's L (experiments only)")
    ap.add_argument("--chunk", type=int, default=0, help="override the workload's chunk (experiments only)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="after the timed region, run a plain device-to-device copy of this many MiB "
                         "(a kernel of known traffic to scale rocprofv3 FETCH_SIZE / WRITE_SIZE by)")
    ap.add_argument("--compare-solvers", action="store_true",
                    help="also time step 2 of Section 3 done by the anti-diagonal sweep of Theorem 3.4 "
                         "(pf_delta_chunk_sigdelta) and report it next to the blocked substitution (flow kernel)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (one MI355X per box); "
              f"--gpus {args.gpus} is not supported. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2504_00492_amd import binding as pf, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    traffic_table = {}
    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(traffic_file):
        try:
            traffic_table = json.load(open(traffic_file))
        except Exception:
            traffic_table = {}

    def workload(name):
        w = synth.WORKLOADS[name]
        if name == args.workload and args.seq_len > 0:
            w = w.with_(L=args.seq_len, name=f"{w.name}@L={args.seq_len}")
        if name == args.workload and args.chunk > 0:
            w = w.with_(chunk=args.chunk, name=f"{w.name}@chunk={args.chunk}")
        return w

    # ---- headline workload
    w = workload(args.workload)
    inputs = device_inputs(synth, w, dev, torch)
    head, O, SL = run_workload(pf, torch, w, inputs, args, traffic_table)
    out = {"metric": "tokens/s, chunked rank-r DeltaNet fwd, 1 MI355X",
           "value": head["value"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": w.dtype, "data": "synthetic"}
    out.update({k: v for k, v in head.items() if k not in out})
    if args.compare_solvers and head["kernels"]:
        out["solvers"] = compare_solvers(pf, torch, w, inputs, head["config"]["flow_block"],
                                         head["kernels"]["flow_kernel"]["ms"], args.steps)
    if args.calibration_copy_mib > 0:
        nbytes = args.calibration_copy_mib << 20
        src = torch.ones(nbytes // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- the oracle on the host cores, on a bounded sample of the headline workload, plus parity on it
    B, H, L, r, dk, dv = w.B, w.H, w.L, w.r, w.d_k, w.d_v
    if not args.no_cpu_baseline:
        import oracle
        cores = min(oracle.max_threads(), os.cpu_count() or 1)
        per_head_flop = (4 * r + 2) * dv * dk * L
        budget_flop = 8e9 * cores            # about ten to twenty seconds of this oracle per core
        nh = int(max(1, min(B * H, budget_flop // per_head_flop)))
        inp = synth.make_inputs(w, list(range(nh)))
        tc0 = time.perf_counter()
        Oref, SLref = oracle.delta_fwd(inp["Q"], inp["K"], inp["V"], inp["beta"], inp["S0"], nthreads=cores)
        tc = time.perf_counter() - tc0
        Og = O.reshape(B * H, L, dv)[:nh].float().cpu().numpy().astype(np.float64)
        Sg = SL.reshape(B * H, dv, dk)[:nh].cpu().numpy().astype(np.float64)
        rel = lambda x, ref: float(np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-300))
        out["cpu_baseline"] = {
            "value": (nh * L / H) / tc, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{nh} of {B * H} (b,h) heads of {w.name}, full L={L}, fp64 token-by-token recurrence; "
                      f"{tc:.2f} s wall; tokens/s scaled as token-heads/s / H",
            "token_heads_per_s": nh * L / tc,
        }
        out["parity_on_sample"] = {"rel_l2_O": rel(Og, Oref), "rel_l2_S_L": rel(Sg, SLref),
                                   "norm_S_L": float(np.linalg.norm(SLref)), "max_abs_O": float(np.abs(Oref).max())}
        del inp, Oref, SLref
    del O, SL

    # ---- every other configuration, each with its own K timed steps
    if not args.only:
        out["configs"] = []
        kept_name, kept = w.name, inputs
        for name in ALL_WORKLOADS:
            if name == args.workload:
                continue
            wi = workload(name)
            same = (synth.WORKLOADS.get(kept_name) is not None and
                    wi.with_(chunk=0, name="") == synth.WORKLOADS[kept_name].with_(chunk=0, name=""))
            if not same:
                del kept
                inputs = None
                torch.cuda.empty_cache()
                kept_name, kept = name, device_inputs(synth, wi, dev, torch)
            res, _, _ = run_workload(pf, torch, wi, kept, args, traffic_table)
            out["configs"].append(res)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
