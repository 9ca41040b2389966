"""bench.py's work and traffic yardsticks against hand-computed values (CPU only).

F_alg per token-head = Gram d r^2 (C-1) + forward substitution for W and U 2 d r^2 (C-1)
+ the three state products (4r+2) d^2 + masked Q K^T and P U_eff d r (C+1) each; minimal HBM
bytes per token-head = read q, r k, r v, r beta and write o."""
import importlib.util
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    try:
        spec.loader.exec_module(mod)
    except ImportError as e:           # the binding needs libpf.so; the formulas do not
        pytest.skip(f"bench.py not importable here: {e}")
    return mod


@pytest.mark.parametrize("d,r,C,f_alg,bytes_bf16", [
    (64, 1, 64, 44992, 514),          # config 1
    (128, 2, 64, 293888, 1540),       # config 2
    (128, 4, 64, 748544, 2568),       # config 3, chunk 64
    (128, 4, 128, 1207296, 2568),     # config 3, chunk 128
    (128, 2, 128, 424960, 1540),      # config 4
])
def test_yardsticks(bench, d, r, C, f_alg, bytes_bf16):
    assert bench.flops_per_token_head(d, r, C) == f_alg
    assert bench.min_bytes_per_token_head(d, r, 2) == bytes_bf16
    # hand count, term by term
    gram = d * r * r * (C - 1)
    solve = 2 * d * r * r * (C - 1)
    state = (4 * r + 2) * d * d
    masked = 2 * d * r * (C + 1)
    assert gram + solve + state + masked == f_alg
    flow, scan = bench.kernel_flops_per_token_head(d, r, C)
    assert flow == gram + d * r * (C + 1)
    assert scan == state + d * r * r * C + d * r * (C + 1)
    bflow, bscan = bench.kernel_bytes_per_token_head(d, r, 2)
    assert bscan == bytes_bf16 and bflow == 2 * d * (1 + r) + 2 * r


def test_config0_fp32_yardsticks(bench):
    assert bench.flops_per_token_head(16, 1, 16) == 2800
    assert bench.min_bytes_per_token_head(16, 1, 4) == 260


@pytest.mark.parametrize("d,r,C,f_dense", [
    (16, 1, 16, 4096),                # config 0
    (64, 1, 64, 65536),               # config 1
    (128, 2, 64, 425984),             # config 2
    (128, 4, 64, 1212416),            # config 3, chunk 64
    (128, 4, 128, 2129920),           # config 3, chunk 128
    (128, 2, 128, 688128),            # config 4
])
def test_full_tile_count(bench, d, r, C, f_dense):
    assert bench.dense_flops_per_token_head(d, r, C) == f_dense
    assert bench.dense_flops_per_token_head(d, r, C) > bench.flops_per_token_head(d, r, C)
