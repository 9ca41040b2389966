"""Seeded sweep over shapes of the MFMA path: random (d, r, chunk, B, H, L, S0, near-reflections,
additive or product form), lengths picked around the flow block (one short of it, exactly it, one
more, several blocks with and without a ragged tail, long enough for the segment-parallel scan).
Every case element by element against the fp64 oracle, through the C ABI, bar 2e-2 (bf16)."""
import random
import sys

import numpy as np
import pytest

from paper_2504_00492_amd import synth
from gpu_util import rel_l2, to_device, flat_heads

pytestmark = pytest.mark.gpu


def test_seeded_shape_sweep(oracle):
    import torch
    from paper_2504_00492_amd import binding as pf
    rng = random.Random(5)
    done = 0
    for it in range(70):
        d = rng.choice([64, 128])
        r = rng.choice([1, 2, 4])
        chunk = rng.choice([32, 64, 128, 256])
        if pf.pf_delta_fwd_supported(d, d, r, chunk, pf.PF_BF16) != 2:
            continue
        blk = pf.pf_delta_fwd_block(d, d, r, chunk, pf.PF_BF16)
        B, H = rng.choice([1, 2]), rng.choice([1, 2, 3, 5])
        L = rng.choice([blk - 1, blk, blk + 1, 3 * blk, 3 * blk + rng.randrange(1, blk), 7 * blk + 5,
                        40 * blk if B * H <= 2 else 5 * blk])
        product = rng.random() < 0.4
        w = synth.Workload("sweep", "bf16", B, H, L, d, d, r, chunk, seed=100 + it,
                           s0_std=rng.choice([0.0, 0.2]), reflect_frac=rng.choice([0.0, 0.1]))
        print(f"[case] sweep {it}: d={d} r={r} chunk={chunk} block={blk} B={B} H={H} L={L} product={product} "
              f"s0={w.s0_std} reflect={w.reflect_frac}", flush=True)
        sys.stdout.flush()
        inp = synth.make_inputs(w)
        dev = to_device(w, inp)
        O, SL = pf.delta_fwd(dev["Q"], dev["K"], dev["V"], dev["beta"], dev["S0"], chunk=chunk, product=product)
        torch.cuda.synchronize()
        ref = oracle.delta_product_fwd if product else oracle.delta_fwd
        Oref, SLref = ref(inp["Q"], inp["K"], inp["V"], inp["beta"], inp["S0"])
        eO = rel_l2(flat_heads(O.float().cpu().numpy()), Oref)
        eS = rel_l2(flat_heads(SL.cpu().numpy()), SLref)
        assert np.isfinite(eO) and eO <= 2e-2 and eS <= 2e-2, (it, eO, eS)
        done += 1
    assert done >= 40
