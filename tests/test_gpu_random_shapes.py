"""Seeded random shapes through the three device calls, each against the oracle:
geometry, group size, element type, stream lengths, budgets, window and pooling
widths are drawn together, so that combinations no hand-written case lists are hit."""
import numpy as np
import pytest

from test_gpu_attend import run_case
from test_gpu_prefill import run_prefill

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", range(12))
def test_random_decode_shapes(xkv, seed):
    r = np.random.default_rng(1000 + seed)
    dtype, d = [("f32", 64), ("bf16", 128), ("bf16", 64), ("f32", 128)][int(r.integers(4))]
    G = int(r.choice([1, 2, 4, 8]))
    Hkv = int(r.integers(1, 4))
    L, B = int(r.integers(1, 4)), int(r.integers(1, 4))
    top = int(r.choice([40, 300, 1200, 5000]))
    lens = r.integers(0, top, size=(L, B))
    append = bool(r.integers(2))
    print(f"decode seed={seed} dtype={dtype} d={d} G={G} Hkv={Hkv} L={L} B={B} lens={lens.tolist()} append={append}",
          flush=True)
    run_case(xkv, dtype, d, Hkv * G, Hkv, L, B, lens, append, seed=2000 + seed, paths=(0, 2))


@pytest.mark.parametrize("seed", range(10))
def test_random_prefill_shapes(xkv, seed):
    r = np.random.default_rng(3000 + seed)
    dtype, d = [("f32", 64), ("bf16", 128), ("bf16", 64), ("f32", 128)][int(r.integers(4))]
    G = int(r.choice([1, 2, 4, 8]))
    Hkv = int(r.integers(1, 3))
    L, B = int(r.integers(1, 3)), int(r.integers(1, 3))
    t = int(r.choice([17, 100, 1000, 2049, 9000]))
    ows = int(min(r.integers(1, 9), 64 // G, t))
    ps = int(r.choice([1, 3, 7]))
    budgets = r.integers(ows, t + 10, size=(L, B))
    print(f"prefill seed={seed} dtype={dtype} d={d} G={G} Hkv={Hkv} L={L} B={B} t={t} ows={ows} ps={ps} "
          f"budgets={budgets.tolist()}", flush=True)
    run_prefill(xkv, dtype, d, Hkv * G, Hkv, L, B, t, ows, ps, budgets, seed=4000 + seed)
