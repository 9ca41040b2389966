#!/usr/bin/env python3
"""Benchmark of the chunked rank-r delta-rule forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2]

One "step" is one pass of the whole hot path (chunk flow + state scan with fused readout, i.e.
one pf_delta_fwd call) over one batch of seeded synthetic input that is already resident in
HBM.  Prints ONE JSON line: tokens/s for the whole job, plus
  * "roofline": the dominant kernel against the roofline that bounds it.  Both kernels sit on the
    HBM side of the ridge (arithmetic intensity about 50-120 flop/B against 2500 TFLOP/s /
    8 TB/s = 312 flop/B), so it is algorithmic bytes (the q, k, v, beta it must read and the o
    it must write) per second against the 8 TB/s HBM peak; the kernel's average duration is
    taken live with HIP events on the launch stream.  Its algorithmic TFLOP/s against the bf16
    MFMA peak is reported next to it ("kernels");
  * "cpu_baseline": the fp64 oracle (oracle/, untuned) timed on this machine's host cores on a
    stated sample of the same workload.
Only one GPU is used; --gpus N with N > 1 exits with a message.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_F32_VALU_TFLOPS = 157.3   # MI355X fp32 vector, published
SETTLE_S = 0.15                # untimed busy time before any timed region (clock settling)
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published


def flops_per_token_head(d, r, C):
    """Headline yardstick: algorithmic (masked, useful) FLOPs per token-head of the chunked
    algorithm with flow blocks of C tokens: Gram d r^2 (C-1), forward substitution for W and U
    2 d r^2 (C-1), the three state products (4r+2) d^2, masked Q K^T and P U_eff d r (C+1) each."""
    return 3 * d * r * r * (C - 1) + (4 * r + 2) * d * d + 2 * d * r * (C + 1)


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # Defaults long enough for the clocks to settle: on this GPU the first few milliseconds of a
    # burst of launches run up to 20 % slower than the steady state (20 steps after 5: 0.277 ms per
    # step on config 2; 400 after 100: 0.23 ms).
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="cfg2",
                    help="cfg0, cfg1, cfg2, cfg3a, cfg3b, cfg4 (see paper_2504_00492_amd/synth.py)")
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
    w = synth.WORKLOADS[args.workload]
    if args.seq_len > 0:
        w = w.with_(L=args.seq_len, name=f"{w.name}@L={args.seq_len}")
    if args.chunk > 0:
        w = w.with_(chunk=args.chunk, name=f"{w.name}@chunk={args.chunk}")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    dt = pf.PF_BF16 if w.dtype == "bf16" else pf.PF_F32
    fam = pf.pf_delta_fwd_supported(w.d_k, w.d_v, w.r, w.chunk, dt)
    if fam == 0:
        print(f"bench.py: no kernel instance for workload {w.name}", file=sys.stderr)
        sys.exit(4)

    # ---- inputs: generated head by head on the host, uploaded once, resident before timing
    B, H, L, r, dk, dv, C = w.B, w.H, w.L, w.r, w.d_k, w.d_v, w.chunk
    Q = torch.empty((B * H, L, dk), dtype=tdt, device=dev)
    K = torch.empty((B * H, L, r, dk), dtype=tdt, device=dev)
    V = torch.empty((B * H, L, r, dv), dtype=tdt, device=dev)
    beta = torch.empty((B * H, L, r), dtype=tdt, device=dev)
    S0 = torch.empty((B * H, dv, dk), dtype=torch.float32, device=dev) if w.s0_std > 0 else None
    for h in range(B * H):
        q, k, v, b, s0 = synth.head_inputs(w, h)
        Q[h] = torch.from_numpy(q).to(dev).to(tdt)
        K[h] = torch.from_numpy(k).to(dev).to(tdt)
        V[h] = torch.from_numpy(v).to(dev).to(tdt)
        beta[h] = torch.from_numpy(b).to(dev).to(tdt)
        if S0 is not None:
            S0[h] = torch.from_numpy(s0).to(dev)
    shp = lambda t: t.reshape((B, H) + tuple(t.shape[1:]))
    Q, K, V, beta = shp(Q), shp(K), shp(V), shp(beta)
    S0 = None if S0 is None else shp(S0)
    O = torch.empty((B, H, L, dv), dtype=tdt, device=dev)
    SL = torch.empty((B, H, dv, dk), dtype=torch.float32, device=dev)
    need = pf.pf_delta_fwd_workspace_bytes(B, H, L, dk, dv, r, C, dt)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    # A small workload would sit in the 256 MB last-level cache if every step read the same
    # buffers: rotate over enough copies of the inputs that each step finds its inputs cold.
    in_bytes = sum(t.numel() * t.element_size() for t in (Q, K, V, beta))
    nsets = 1 if in_bytes >= 256 * 2 ** 20 else min(64, -(-(600 * 2 ** 20) // in_bytes))
    sets = [(Q, K, V, beta)] + [tuple(t.clone() for t in (Q, K, V, beta)) for _ in range(nsets - 1)]

    def step(i=0):
        q, k, v, b = sets[i % nsets]
        st = pf.pf_delta_fwd(q, k, v, b, S0, O, SL, B, H, L, dk, dv, r, C, dt, ws, need, stream)
        if st != pf.PF_OK:
            raise pf.PfError(st, "pf_delta_fwd")

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # Whatever W is, keep warming up (untimed) until the GPU has been busy for SETTLE_S seconds:
    # the clocks need that long to settle (see the defaults above), and a short W would time the
    # transient instead of the throughput of the job.
    settle_steps = 0
    ts = time.perf_counter()
    while time.perf_counter() - ts < SETTLE_S and settle_steps < 20000:
        for i in range(20):
            step(args.warmup + settle_steps + i)
        settle_steps += 20
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step(0)                      # leave the outputs of input set 0 behind for the parity check
    torch.cuda.synchronize()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens = B * L
    token_heads = B * H * L
    tok_per_s = tokens / (ms_per_step * 1e-3)

    # flow block: the requested chunk unless chunk * r virtual tokens exceed a kernel instance
    block = pf.pf_delta_fwd_block(dk, dv, r, C, dt) if fam == 2 else C
    f_alg = flops_per_token_head(dk, r, block)
    f_flow, f_scan = kernel_flops_per_token_head(dk, r, block)
    e = 2 if w.dtype == "bf16" else 4
    min_bytes = min_bytes_per_token_head(dk, r, e) * token_heads
    b_flow, b_scan = kernel_bytes_per_token_head(dk, r, e)

    # ---- per-kernel durations, HIP events on the launch stream (same kernels, same arguments)
    kernels = {}
    if fam == 2:
        n = block * r
        NC = L // block
        mk = lambda m: torch.empty((B, H, NC, m), dtype=torch.bfloat16, device=dev)
        Tt, Pt = mk(n * n), mk(block * n)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
        nwarm = args.warmup + settle_steps
        for i in range(nwarm + args.steps):
            j = i - nwarm
            if j >= 0:
                ev[j][0].record(stream)
            st = pf.pf_delta_chunk_flow(Q, K, beta, Tt, Pt, B, H, L, dk, dv, r, block, stream)
            assert st == pf.PF_OK, st
            if j >= 0:
                ev[j][1].record(stream)
            st = pf.pf_delta_chunk_scan(Q, K, V, beta, Tt, Pt, S0, O, SL, B, H, L, dk, dv, r, block, stream)
            assert st == pf.PF_OK, st
            if j >= 0:
                ev[j][2].record(stream)
        torch.cuda.synchronize()
        t_flow = sum(a.elapsed_time(b) for a, b, _ in ev) / args.steps
        t_scan = sum(b.elapsed_time(c) for _, b, c in ev) / args.steps
        def kinfo(ms, fl, by):
            tf = fl * token_heads / (ms * 1e-3) / 1e12
            gb = by * token_heads / (ms * 1e-3) / 1e9
            return {"ms": ms, "alg_tflops": tf, "frac_bf16_mfma_peak": tf / PEAK_BF16_TFLOPS,
                    "alg_gbs": gb, "frac_hbm_peak": gb / PEAK_HBM_GBS,
                    "alg_bytes_per_launch": by * token_heads, "flop_per_alg_byte": fl / by}
        kernels = {"flow_kernel": kinfo(t_flow, f_flow, b_flow), "scan_kernel": kinfo(t_scan, f_scan, b_scan)}
        dom = "flow_kernel" if t_flow >= t_scan else "scan_kernel"
        roofline = {"bound": "hbm", "kernel": dom, "achieved": kernels[dom]["alg_gbs"],
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": kernels[dom]["frac_hbm_peak"],
                    "avg_kernel_ms": kernels[dom]["ms"], "traffic": None}
    else:
        tfl = f_alg * token_heads / (ms_per_step * 1e-3) / 1e12
        roofline = {"bound": "alu", "kernel": "generic_kernel", "achieved": tfl, "peak": PEAK_F32_VALU_TFLOPS,
                    "unit": "TFLOP/s", "frac": tfl / PEAK_F32_VALU_TFLOPS, "avg_kernel_ms": ms_per_step,
                    "traffic": None}
    solvers = None
    if args.compare_solvers and pf.pf_delta_chunk_sigdelta_supported(dk, dv, r, block, dt):
        Cs = block                       # both solvers on the same blocks
        sneed = pf.pf_delta_chunk_sigdelta_workspace_bytes(B, H, L, r, Cs)
        sws = torch.empty(sneed, dtype=torch.uint8, device=dev)
        Wo = torch.empty((B, H, L, r, dk), dtype=torch.float32, device=dev)
        Uo = torch.empty((B, H, L, r, dv), dtype=torch.float32, device=dev)
        nrep = min(10, max(3, args.steps // 4))
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(nrep)]
        for i in range(1 + nrep):
            if i >= 1:
                evs[i - 1][0].record(stream)
            st = pf.pf_delta_chunk_sigdelta(K, V, beta, Wo, Uo, B, H, L, dk, dv, r, Cs, dt, sws, sneed, stream)
            assert st == pf.PF_OK, st
            if i >= 1:
                evs[i - 1][1].record(stream)
        torch.cuda.synchronize()
        t_sig = sum(a.elapsed_time(b) for a, b in evs) / nrep
        n_sig = Cs * r
        # useful fp32 operations of the sweep: C(C-1)/2 grid cells, r rows of d_k + d_v columns, 2 + r
        # additions / multiply-adds each (counted as 2 flops), per chunk-head
        sig_flops = (Cs * (Cs - 1) // 2) * r * (dk + dv) * (2 + r) * 2 * (token_heads / Cs)
        solvers = {
            "sigdelta": {"ms": t_sig, "chunk": Cs, "n": n_sig, "gives": "W, U fp32 (Gram kernel + sweep kernel)",
                         "sweep_tflops_fp32": sig_flops / (t_sig * 1e-3) / 1e12,
                         "frac_fp32_valu_peak": sig_flops / (t_sig * 1e-3) / 1e12 / PEAK_F32_VALU_TFLOPS},
            "block_substitution": {"ms": kernels.get("flow_kernel", {}).get("ms"), "chunk": block, "n": block * r,
                                   "gives": "T = (Id + G)^-1 and P, bf16 (W = T beta K and U are formed by "
                                            "the scan kernel)"},
        }
        del sws, Wo, Uo
    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(traffic_file):
        try:
            roofline["traffic"] = json.load(open(traffic_file)).get(w.name, {}).get(roofline["kernel"])
        except Exception:
            pass

    if args.calibration_copy_mib > 0:
        nbytes = args.calibration_copy_mib << 20
        src = torch.ones(nbytes // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    alg_tflops = f_alg * token_heads / (ms_per_step * 1e-3) / 1e12
    out = {
        "metric": "tokens/s, chunked rank-r DeltaNet fwd, 1 MI355X",
        "value": tok_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_steps": settle_steps,   # further untimed steps after the W warm-up steps (>= 0.15 s of GPU work)
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: B={B} H={H} L={L} d_k=d_v={dk} r={r} chunk={C} {w.dtype}",
                   "kernel_family": {1: "generic", 2: "mfma"}[fam], "flow_block": block},
        "alg_tflops": alg_tflops, "frac_bf16_mfma_peak": alg_tflops / PEAK_BF16_TFLOPS,
        # the same time priced with the flop count of the requested chunk (what a run blocked at
        # that chunk would have executed); equal to alg_tflops when flow_block == chunk
        "alg_tflops_at_requested_chunk": flops_per_token_head(dk, r, C) * token_heads / (ms_per_step * 1e-3) / 1e12,
        "token_heads_per_s": token_heads / (ms_per_step * 1e-3),
        "min_hbm_gbs": min_bytes / (ms_per_step * 1e-3) / 1e9,
        "frac_hbm_peak_min_traffic": min_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "kernels": kernels, "roofline": roofline,
        # inputs + outputs + workspace of one step; when that is below the 256 MB last-level cache
        # the inputs are rotated over several copies so that each step reads them from HBM
        "working_set_bytes": int(min_bytes + need + B * H * dv * dk * 4),
        "cache_resident": bool(min_bytes + need + B * H * dv * dk * 4 < 256 * 2 ** 20) and nsets == 1,
        "input_sets_rotated": nsets,
    }
    if solvers is not None:
        out["solvers"] = solvers

    # ---- the oracle on the host cores, on a bounded sample of the same workload, plus parity on it
    if not args.no_cpu_baseline:
        import oracle
        cores = min(oracle.max_threads(), os.cpu_count() or 1)
        per_head_flop = (4 * r + 2) * dv * dk * L
        budget_flop = 8e9 * cores            # about ten seconds of this oracle per core
        nh = int(max(1, min(B * H, budget_flop // per_head_flop)))
        heads = list(range(nh))
        inp = synth.make_inputs(w, heads)
        tc0 = time.perf_counter()
        Oref, SLref = oracle.delta_fwd(inp["Q"], inp["K"], inp["V"], inp["beta"], inp["S0"], nthreads=cores)
        tc = time.perf_counter() - tc0
        Og = O.reshape(B * H, L, dv)[:nh].float().cpu().numpy().astype(np.float64)
        Sg = SL.reshape(B * H, dv, dk)[:nh].cpu().numpy().astype(np.float64)
        rel = lambda x, ref: float(np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-300))
        out["cpu_baseline"] = {
            "value": (nh * L / H) / tc, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{nh} of {B * H} (b,h) heads, full L={L}, fp64 token-by-token recurrence; "
                      f"{tc:.2f} s wall; tokens/s scaled as token-heads/s / H",
            "token_heads_per_s": nh * L / tc,
        }
        out["parity_on_sample"] = {"rel_l2_O": rel(Og, Oref), "rel_l2_S_L": rel(Sg, SLref),
                                   "norm_S_L": float(np.linalg.norm(SLref)), "max_abs_O": float(np.abs(Oref).max())}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
