"""GPU parity: xkv_evict_compact against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

from oracle import xkv_oracle as orc
from gpu_util import get_unit, random_fill

pytestmark = pytest.mark.gpu


def run_case(xkv, dtype, d, Hkv, L, B, lens, budgets, pool, protect, seed, ties, with_kept=True,
             layer_range=None, pos_sequential=False):
    lens = np.asarray(lens, np.int32).reshape(L, B)
    cache = xkv.XkvCache(L, B, Hkv, Hkv, d, dtype, lens + 1)
    random_fill(cache, lens, seed, ties=ties)
    if pos_sequential:
        for l in range(L):
            for b in range(B):
                for h in range(Hkv):
                    s0 = cache.stream_slot(l, b, h)
                    cache.pos[s0:s0 + lens[l, b]] = torch.arange(lens[l, b], dtype=torch.int32, device="cuda")
    l0, l1 = layer_range or (0, L)
    budgets = np.asarray(budgets, np.int32).reshape(l1 - l0, B)
    before = {(l, b, h): get_unit(cache, l, b, h) for l in range(L) for b in range(B) for h in range(Hkv)}
    kept = torch.full((cache.arena_slots,), -7, dtype=torch.int32, device="cuda") if with_kept else None
    ws = torch.empty(xkv.xkv_workspace_bytes(cache, L), dtype=torch.uint8, device="cuda")
    xkv.xkv_evict_compact(cache, l0, l1, budgets, ws, pool_size=pool, n_protect=protect, kept_idx_out=kept)
    torch.cuda.synchronize()
    for (l, b, h), (K, V, score, pos) in before.items():
        if not (l0 <= l < l1):
            assert cache.length(l, b) == lens[l, b]
            continue
        bud = int(budgets[l - l0, b])
        K2, V2, s2, p2, kept_idx = orc.evict_compact(K, V, score, pos, bud, pool, protect)
        kk = min(bud, int(lens[l, b]))
        assert cache.length(l, b) == kk
        gK, gV, gs, gp = get_unit(cache, l, b, h)
        tag = f"unit {(l, b, h)} n={lens[l, b]} k={bud}"
        if with_kept:
            s0 = cache.stream_slot(l, b, h)
            assert np.array_equal(kept[s0:s0 + kk].cpu().numpy(), kept_idx), tag
        assert np.array_equal(gp, p2), tag
        assert np.array_equal(gs, s2), tag
        assert np.array_equal(gK, K2) and np.array_equal(gV, V2), tag
        # slots past the new length keep whatever they held: the stream's capacity is untouched


@pytest.mark.parametrize("ties", [False, True])
@pytest.mark.parametrize("pool,protect", [(1, 0), (7, 0), (1, 8), (7, 8), (3, 1)])
def test_selection_and_compaction(xkv, ties, pool, protect):
    lens = [[1, 9], [64, 511], [512, 513], [1500, 4100]]
    budgets = np.maximum(np.array([[1, 8], [20, 300], [511, 100], [1499, 1000]]), protect)
    print(f"case ties={ties} pool={pool} protect={protect}", flush=True)
    run_case(xkv, "f32", 64, 2, 4, 2, lens, budgets, pool, protect, seed=1, ties=ties,
             pos_sequential=protect > 0)


def test_degenerate_budgets(xkv):
    lens = [[100, 100, 100, 0]]
    run_case(xkv, "bf16", 128, 2, 1, 4, lens, [[100, 500, 0, 3]], 1, 0, seed=2, ties=False)
    run_case(xkv, "bf16", 128, 2, 1, 4, lens, [[99, 1, 50, 0]], 1, 0, seed=3, ties=True)


def test_all_scores_equal_keeps_the_first_slots(xkv):
    cache = xkv.XkvCache(1, 1, 1, 1, 64, "f32", [[1000]])
    random_fill(cache, [[1000]], 4)
    cache.score.fill_(0.25)
    kept = torch.zeros(cache.arena_slots, dtype=torch.int32, device="cuda")
    ws = torch.empty(xkv.xkv_workspace_bytes(cache, 1), dtype=torch.uint8, device="cuda")
    xkv.xkv_evict_compact(cache, 0, 1, np.array([[600]], np.int32), ws, kept_idx_out=kept)
    torch.cuda.synchronize()
    assert np.array_equal(kept[:600].cpu().numpy(), np.arange(600))


def test_large_moves_use_the_separate_move_kernel(xkv):
    """Thousands of rows to move per stream, several dtypes / row sizes."""
    for dtype, d in (("bf16", 128), ("f32", 128), ("bf16", 64)):
        print(f"case big moves {dtype} {d}", flush=True)
        run_case(xkv, dtype, d, 2, 2, 1, [[9000], [33000]], [[3000], [6500]], 1, 0, seed=5, ties=False)
    run_case(xkv, "bf16", 128, 1, 1, 1, [[20000]], [[10000]], 7, 8, seed=6, ties=True, pos_sequential=True)


def test_steady_state_single_eviction_and_subrange(xkv):
    run_case(xkv, "bf16", 128, 4, 3, 2, [[301, 33], [1001, 2049], [77, 5000]],
             [[1000, 2048]], 1, 0, seed=7, ties=False, layer_range=(1, 2))
    run_case(xkv, "bf16", 128, 4, 3, 2, [[301, 33], [1001, 2049], [77, 5000]],
             [[300, 32], [1000, 2048], [76, 4999]], 1, 0, seed=8, ties=True, with_kept=False)


@pytest.mark.parametrize("pool,protect,top", [(1, 0, 300), (7, 8, 300), (1, 0, 3000)])
def test_more_regions_than_the_kernel_arguments_hold(xkv, pool, protect, top):
    """More than 128 regions: the region table goes through device memory and the call is one
    selection launch (plus the move launch when streams move many rows, top = 3000)."""
    L, B = 3, 70
    r = np.random.default_rng(1 + top)
    lens = r.integers(1, top, size=(L, B))
    budgets = np.maximum(max(1, protect), (lens * r.random((L, B))).astype(np.int32))
    run_case(xkv, "bf16", 64, 2, L, B, lens, budgets, pool, protect, seed=9, ties=True)
    # steady state of decoding: one eviction per stream
    run_case(xkv, "f32", 64, 1, L, B, lens, np.maximum(lens - 1, max(1, protect)), pool, protect, seed=10, ties=False)


@pytest.mark.parametrize("pool,protect", [(1, 0), (7, 8)])
def test_few_evictions_per_stream(xkv, pool, protect):
    """Between 0 and 8 evictions per stream (the steady state of decoding evicts one),
    with ties, including the case where the newest slots are themselves evicted."""
    lens = np.array([[40, 600], [513, 2049], [1025, 9], [300, 4100]])
    drop = np.array([[0, 1], [2, 8], [5, 3], [8, 7]])
    for ties in (True, False):
        print(f"case few evictions ties={ties} pool={pool} protect={protect}", flush=True)
        run_case(xkv, "bf16", 128, 2, 4, 2, lens, np.maximum(lens - drop, protect), pool, protect, seed=11, ties=ties,
                 pos_sequential=protect > 0)
