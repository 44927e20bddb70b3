"""GPU parity: the device allocator against the oracle's Alg. 1, and the
mini-prefill's attention processing (xkv_window_importance) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import xkv_oracle as orc
from gpu_util import TOL, rel_err, storage
import xkv_workloads as wl

pytestmark = pytest.mark.gpu


def device_allocate(xkv, curves, total, lo=None, hi=None, stride=None):
    L, T = curves.shape
    stride = stride or T
    buf = torch.zeros((L, stride), dtype=torch.float32)
    buf[:, :T] = torch.from_numpy(curves)
    buf = buf.cuda()
    ws = torch.empty(xkv.xkv_allocate_device_workspace_bytes(L, T), dtype=torch.uint8, device="cuda")
    return xkv.xkv_allocate_budgets_device(buf, L, T, stride, total, ws, lo, hi)


def check_optimal(curves, n, lo, hi):
    """Exchange invariant: no evicted value of a layer below its cap beats a kept
    value of a layer above its floor (contributions in float64)."""
    L, T = curves.shape
    worst_kept, best_out = np.inf, -np.inf
    for l in range(L):
        s = np.sort(curves[l].astype(np.float64))[::-1]
        tot = s.sum()
        p = s / tot if tot > 0 else np.zeros_like(s)
        if n[l] > lo[l]:
            worst_kept = min(worst_kept, p[n[l] - 1])
        if n[l] < hi[l]:
            best_out = max(best_out, p[n[l]])
    assert best_out <= worst_kept * (1 + 1e-12) + 1e-300


@pytest.mark.parametrize("L,T,frac", [(4, 1000, 0.3), (32, 4096, 0.4), (7, 20001, 0.15), (3, 50, 0.9)])
def test_matches_the_oracle_on_zipf_curves(xkv, L, T, frac):
    curves = np.stack(wl.zipf_importance_curves(L, T, seed=11 + L))
    total = int(frac * L * T)
    got, ravg = device_allocate(xkv, curves, total)
    ref, ravg_ref = orc.allocate_budgets([c for c in curves], total_size=total)
    assert got.sum() == total
    assert np.array_equal(got, np.asarray(ref)), (got, ref)
    assert abs(ravg - ravg_ref) < 1e-9


def test_floors_caps_and_stride(xkv):
    r = np.random.default_rng(5)
    for trial in range(6):
        L, T = int(r.integers(2, 12)), int(r.integers(40, 3000))
        curves = (r.random((L, T)) ** r.uniform(1, 6, size=(L, 1))).astype(np.float32)
        lo = r.integers(0, T // 4, size=L).astype(np.int64)
        hi = np.minimum(T, lo + r.integers(1, T, size=L)).astype(np.int64)
        total = int(r.integers(lo.sum(), hi.sum() + 1))
        got, ravg = device_allocate(xkv, curves, total, lo, hi, stride=T + 13)
        ref, ravg_ref = orc.allocate_budgets([c for c in curves], total_size=total, min_budget=lo, max_budget=hi)
        assert got.sum() == total and np.all(got >= lo) and np.all(got <= hi)
        check_optimal(curves, got, lo, hi)
        assert abs(ravg - ravg_ref) < 1e-9, (trial, ravg, ravg_ref)
        assert np.array_equal(got, np.asarray(ref)), (trial, got, ref)


def test_ties_and_zero_layers(xkv):
    """Identical layers tie everywhere: the lower layers are served first; a layer
    of zeros receives tokens only when nothing else is left."""
    T = 64
    base = np.linspace(1.0, 2.0, T).astype(np.float32)
    curves = np.stack([base, base, np.zeros(T, np.float32), base])
    for total in (1, 2, 3, 50, 3 * T, 3 * T + 5, 4 * T):
        got, ravg = device_allocate(xkv, curves, total)
        ref, ravg_ref = orc.allocate_budgets([c for c in curves], total_size=total)
        assert np.array_equal(got, np.asarray(ref)), (total, got, ref)
        assert abs(ravg - ravg_ref) < 1e-12
    got, _ = device_allocate(xkv, curves, 0)
    assert not got.any()


def test_full_size_config_matches_the_oracle(xkv):
    """32 x 32768 curves of the long-context workload: device result = the oracle's
    (and the host library's, which has its own test against the oracle)."""
    w = wl.WORKLOADS["llama2_7b_32k"]
    curves = np.stack(wl.zipf_importance_curves(w.n_layers, w.context, seed=w.seed))
    got, ravg = device_allocate(xkv, curves, w.total_budget)
    ref, ravg_ref = orc.allocate_budgets([c for c in curves], total_size=w.total_budget)
    assert np.array_equal(got, np.asarray(ref)) and abs(ravg - ravg_ref) < 1e-9
    host, ravg_host = xkv.xkv_allocate_budgets([c for c in curves], total_size=w.total_budget)
    assert np.array_equal(got, host) and abs(ravg - ravg_host) < 1e-9


@pytest.mark.parametrize("dtype,d,G,Hkv", [("bf16", 128, 1, 4), ("bf16", 128, 4, 2), ("f32", 64, 2, 3)])
def test_window_importance_then_allocate_then_prefill(xkv, dtype, d, G, Hkv):
    """The mini-prefill flow: score vectors on the device, budgets from the device
    allocator, prefill eviction with those budgets."""
    L, B, t, ows, ps = 3, 2, 900, 8, 7
    Hq = Hkv * G
    tc = t - ows
    cache = xkv.XkvCache(L, B, Hq, Hkv, d, dtype, np.full((L, B), t, np.int32))
    g = torch.Generator(device="cpu").manual_seed(77)
    k_src = torch.randn((L, B, Hkv, t, d), generator=g)
    k_src[:, :, :, ::37, :] *= 3.0
    k_src = k_src.to(cache.torch_dtype).cuda()
    v_src = torch.randn((L, B, Hkv, t, d), generator=g).to(cache.torch_dtype).cuda()
    q_win = torch.randn((L, B, Hq, ows, d), generator=g).to(cache.torch_dtype).cuda()
    ws = torch.empty(xkv.xkv_prefill_workspace_bytes(cache, L, t, ows), dtype=torch.uint8, device="cuda")
    w_layer = torch.full((L, B, tc), float("nan"), dtype=torch.float32, device="cuda")
    xkv.xkv_window_importance(cache, 0, L, q_win, k_src, t, ows, w_layer, ws, pool_size=ps)
    torch.cuda.synchronize()
    wl_host = w_layer.cpu().numpy()
    for l in range(L):
        for b in range(B):
            q = storage(q_win[l, b]).reshape(Hkv, G, ows, d)
            ref = orc.window_importance(q, storage(k_src[l, b]), ps)
            assert rel_err(wl_host[l, b], ref) <= TOL[dtype]
    # per sequence: allocate on the device straight from w_layer (layer stride B * tc)
    total = int(0.3 * L * t)
    aws = torch.empty(xkv.xkv_allocate_device_workspace_bytes(L, tc), dtype=torch.uint8, device="cuda")
    budgets = np.zeros((L, B), np.int32)
    for b in range(B):
        got, ravg = xkv.xkv_allocate_budgets_device(w_layer[:, b], L, tc, B * tc, total - L * ows, aws)
        ref, ravg_ref = orc.allocate_budgets([wl_host[l, b] for l in range(L)], total_size=total - L * ows)
        assert np.array_equal(got, np.asarray(ref)) and abs(ravg - ravg_ref) < 1e-9
        budgets[:, b] = got + ows                       # the window's tokens come on top
    xkv.xkv_prefill_evict(cache, 0, L, q_win, k_src, v_src, t, ows, budgets, ws, pool_size=ps)
    torch.cuda.synchronize()
    assert np.array_equal(cache.len.reshape(L, B), budgets)
    assert int(cache.len.sum()) == B * total


def retained(curves, n):
    """R_avg of an allocation, straight from Eq. 4."""
    return float(np.mean([orc.retention_ratio(curves[l], int(n[l])) for l in range(len(n))]))


@pytest.mark.parametrize("L,T,target", [(4, 1000, 0.5), (16, 3000, 0.8), (6, 20001, 0.93), (3, 50, 1.0), (5, 400, 0.0)])
def test_target_mode_finds_the_smallest_total(xkv, L, T, target):
    """Eq. 18 on the device: R_avg reaches the target, one token less does not; the total agrees
    with the oracle's greedy (exactly, unless R_avg sits on the target to within rounding)."""
    curves = np.stack(wl.zipf_importance_curves(L, T, seed=21 + L))
    buf = torch.from_numpy(curves).cuda()
    ws = torch.empty(xkv.xkv_allocate_device_workspace_bytes(L, T), dtype=torch.uint8, device="cuda")
    got, ravg = xkv.xkv_allocate_budgets_device(buf, L, T, T, 0, ws, mode=xkv.XKV_ALLOC_TARGET_RAVG,
                                                target_ravg=target)
    ref, ravg_ref = orc.allocate_budgets([c for c in curves], target_ravg=target)
    assert abs(ravg - retained(curves, got)) < 1e-9
    assert ravg >= target - 1e-12
    total = int(got.sum())
    if total > 0:
        less, r_less = xkv.xkv_allocate_budgets_device(buf, L, T, T, total - 1, ws)
        assert r_less < target + 1e-12
    assert abs(total - int(np.sum(ref))) <= 1, (total, int(np.sum(ref)))
    if total == int(np.sum(ref)):
        assert np.array_equal(got, np.asarray(ref))


def test_target_mode_with_floors_and_caps(xkv):
    r = np.random.default_rng(8)
    L, T = 7, 900
    curves = (r.random((L, T)) ** r.uniform(1, 5, size=(L, 1))).astype(np.float32)
    lo = r.integers(0, 100, size=L).astype(np.int64)
    hi = (lo + r.integers(50, 700, size=L)).astype(np.int64)
    buf = torch.from_numpy(curves).cuda()
    ws = torch.empty(xkv.xkv_allocate_device_workspace_bytes(L, T), dtype=torch.uint8, device="cuda")
    for target in (0.3, 0.7, 0.999):
        got, ravg = xkv.xkv_allocate_budgets_device(buf, L, T, T, 0, ws, min_budget=lo, max_budget=hi,
                                                    mode=xkv.XKV_ALLOC_TARGET_RAVG, target_ravg=target)
        ref, ravg_ref = orc.allocate_budgets([c for c in curves], target_ravg=target, min_budget=lo, max_budget=hi)
        assert np.all(got >= lo) and np.all(got <= np.minimum(hi, T))
        assert abs(int(got.sum()) - int(np.sum(ref))) <= 1
        if int(got.sum()) == int(np.sum(ref)):
            assert np.array_equal(got, np.asarray(ref)) and abs(ravg - ravg_ref) < 1e-9
