"""Host-side checks of libxkv.so that need no GPU: every symbol of the header
is exported, the allocator agrees with the oracle, and argument errors are
reported before anything touches a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2412_05896_amd as xkv
from paper_2412_05896_amd import binding
from oracle import xkv_oracle as orc
import xkv_workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = xkv.load()
    header = open(os.path.join(ROOT, "include", "xkv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(xkv_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert xkv.status_string(0) == "XKV_OK"
    assert xkv.status_string(-3) == "XKV_ERR_CAPACITY"


# ---- allocator vs oracle --------------------------------------------------
@pytest.mark.parametrize("seed", range(6))
def test_allocator_matches_oracle_total_mode(seed):
    r = np.random.default_rng(seed)
    L = int(r.integers(1, 9))
    w = [np.round(r.random(int(r.integers(1, 400))) ** 4, 3).astype(np.float32) for _ in range(L)]
    lens = [x.size for x in w]
    for N in sorted({0, 1, sum(lens) // 3, sum(lens) // 2, sum(lens) - 1, sum(lens)}):
        got, ravg = xkv.xkv_allocate_budgets(w, total_size=N)
        ref, rref = orc.allocate_budgets(w, total_size=N)
        np.testing.assert_array_equal(got, ref)
        assert abs(ravg - rref) < 1e-12


def test_allocator_floors_caps_and_ties():
    r = np.random.default_rng(42)
    L = 5
    w = [r.integers(0, 4, size=50).astype(np.float32) for _ in range(L)]
    w[2][:] = 0                                   # a layer with no importance at all
    lo = [3, 0, 2, 10, 0]
    hi = [50, 20, 50, 30, 5]
    for N in (15, 16, 40, 99, 155):
        got, ravg = xkv.xkv_allocate_budgets(w, total_size=N, min_budget=lo, max_budget=hi)
        ref, rref = orc.allocate_budgets(w, total_size=N, min_budget=lo, max_budget=hi)
        np.testing.assert_array_equal(got, ref)
        assert abs(ravg - rref) < 1e-12


@pytest.mark.parametrize("seed", range(3))
def test_allocator_matches_oracle_target_mode(seed):
    r = np.random.default_rng(50 + seed)
    w = [r.random(int(r.integers(20, 200))).astype(np.float32) ** 3 for _ in range(4)]
    for target in (0.0, 0.1, 0.5, 0.9, 0.999, 1.0):
        got, ravg = xkv.xkv_allocate_budgets(w, mode=xkv.XKV_ALLOC_TARGET_RAVG, target_ravg=target)
        ref, rref = orc.allocate_budgets(w, target_ravg=target)
        np.testing.assert_array_equal(got, ref)
        assert abs(ravg - rref) < 1e-12
    got, _ = xkv.xkv_allocate_budgets(w, mode=xkv.XKV_ALLOC_TARGET_RAVG, target_ravg=0.5,
                                      min_budget=[5, 0, 1, 0])
    ref, _ = orc.allocate_budgets(w, target_ravg=0.5, min_budget=[5, 0, 1, 0])
    np.testing.assert_array_equal(got, ref)


def test_allocator_on_the_benchmark_curves():
    """Zipf curves of the Llama-2-7B-shaped 4k workload, 40 % total budget."""
    w = wl.WORKLOADS["llama2_7b_4k"]
    curves = wl.zipf_importance_curves(w.n_layers, w.context, w.seed)
    got, ravg = xkv.xkv_allocate_budgets(curves, total_size=w.total_budget)
    ref, rref = orc.allocate_budgets(curves, total_size=w.total_budget)
    np.testing.assert_array_equal(got, ref)
    assert int(got.sum()) == w.total_budget == 52428
    assert abs(ravg - rref) < 1e-12
    assert got.max() > 2 * got.min()              # budgets really differ by layer


def test_allocator_errors():
    w = [np.ones(4, np.float32), np.ones(4, np.float32)]
    E = xkv.XkvError
    for kwargs, code in [
        (dict(total_size=9), -2), (dict(total_size=-1), -2),
        (dict(total_size=3, min_budget=[2, 2]), -2),
        (dict(total_size=3, min_budget=[3, 0], max_budget=[2, 4]), -2),
        (dict(total_size=7, max_budget=[3, 3]), -2),
        (dict(mode=7, total_size=1), -1),
        (dict(mode=xkv.XKV_ALLOC_TARGET_RAVG, target_ravg=1.5), -1),
        (dict(mode=xkv.XKV_ALLOC_TARGET_RAVG, target_ravg=float("nan")), -1),
    ]:
        with pytest.raises(E) as e:
            xkv.xkv_allocate_budgets(w, **kwargs)
        assert e.value.status == code, kwargs
    for bad in (np.nan, np.inf, -1.0):
        with pytest.raises(E) as e:
            xkv.xkv_allocate_budgets([np.array([1.0, bad], np.float32)], total_size=1)
        assert e.value.status == -1
    lib = xkv.load()
    assert lib.xkv_allocate_budgets(0, None, None, 0, 0, 0.0, None, None, None, None) == -1


# ---- descriptor validation (host only: fake, never dereferenced, device pointers) ----
def _fake_cache(**over):
    s = binding._CacheStruct()
    L, B = 2, 2
    keep = {}
    keep["off"] = np.array([0, 400, 800, 1200], np.int64)
    keep["cap"] = np.array([100, 100, 100, 100], np.int32)
    keep["len"] = np.array([10, 20, 30, 100], np.int32)
    s.n_layers, s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim, s.dtype = L, B, 8, 4, 128, 1
    s.arena_slots = 1600
    s.k = s.v = s.score = s.pos = 0x1000       # never dereferenced on an error path
    s.region_off = keep["off"].ctypes.data
    s.cap = keep["cap"].ctypes.data
    s.len = keep["len"].ctypes.data
    for k, v in over.items():
        setattr(s, k, v)
    return s, keep


def test_cache_descriptor_errors():
    lib = xkv.load()
    out = C.c_size_t(0)
    s, keep = _fake_cache()
    assert lib.xkv_workspace_bytes(C.byref(s), 2, C.byref(out)) == 0 and out.value > 0
    assert lib.xkv_workspace_bytes(None, 2, C.byref(out)) == -1
    assert lib.xkv_workspace_bytes(C.byref(s), 0, C.byref(out)) == -1
    for over, code in [(dict(n_q_heads=6), -1), (dict(head_dim=96), -4), (dict(n_q_heads=64), -4),
                       (dict(dtype=5), -1), (dict(k=0), -1), (dict(k=0x1008), -1),
                       (dict(arena_slots=1599), -1), (dict(n_layers=0), -1)]:
        s, keep = _fake_cache(**over)
        assert lib.xkv_workspace_bytes(C.byref(s), 2, C.byref(out)) == code, over
    s, keep = _fake_cache()
    keep["len"][1] = 101                           # len > cap
    assert lib.xkv_workspace_bytes(C.byref(s), 2, C.byref(out)) == -1


def test_attend_and_evict_argument_errors_leave_state_untouched():
    lib = xkv.load()
    s, keep = _fake_cache()
    q = 0x2000
    pos_new = np.zeros(2, np.int32)
    big = 1 << 30
    call = lambda *a: lib.xkv_decode_attend_score(C.byref(s), *a)
    assert call(0, 0, q, q, q, pos_new.ctypes.data, 0.0, q, q, big, None) == -1      # empty range
    assert call(0, 3, q, q, q, pos_new.ctypes.data, 0.0, q, q, big, None) == -1      # past the end
    assert call(0, 2, None, q, q, pos_new.ctypes.data, 0.0, q, q, big, None) == -1   # no q
    assert call(0, 2, q, q, None, pos_new.ctypes.data, 0.0, q, q, big, None) == -1   # k_new without v_new
    assert call(0, 2, q, q, q, None, 0.0, q, q, big, None) == -1                     # append without pos
    assert call(0, 2, q, q, q, pos_new.ctypes.data, -1.0, q, q, big, None) == -1     # negative scale
    assert call(1, 2, q, q, q, pos_new.ctypes.data, 0.0, q, q, big, None) == -3      # stream (1,1) is full
    assert call(0, 1, q, q, q, pos_new.ctypes.data, 0.0, q, q, 16, None) == -3       # workspace too small
    assert keep["len"].tolist() == [10, 20, 30, 100]
    bud = np.array([5, 5, 5, 5], np.int32)
    ev = lambda *a: lib.xkv_evict_compact(C.byref(s), *a)
    assert ev(0, 2, None, 1, 0, None, q, big, None) == -1
    assert ev(0, 2, bud.ctypes.data, 2, 0, None, q, big, None) == -1                 # even pooling width
    assert ev(0, 2, bud.ctypes.data, 1, -1, None, q, big, None) == -1
    assert ev(0, 2, bud.ctypes.data, 1, 6, None, q, big, None) == -1                 # budget < protected
    assert ev(0, 2, bud.ctypes.data, 1, 0, None, q, 8, None) == -3
    neg = np.array([5, -1, 5, 5], np.int32)
    assert ev(0, 2, neg.ctypes.data, 1, 0, None, q, big, None) == -1
    assert keep["len"].tolist() == [10, 20, 30, 100]


def test_prefill_argument_errors_leave_state_untouched():
    lib = xkv.load()
    s, keep = _fake_cache()                      # G = 2, caps 100
    p = 0x2000
    big = 1 << 30
    bud = np.array([50, 50, 50, 50], np.int32)
    out = C.c_size_t(0)
    assert lib.xkv_prefill_workspace_bytes(C.byref(s), 2, 300, 8, C.byref(out)) == 0 and out.value > 0
    assert lib.xkv_prefill_workspace_bytes(C.byref(s), 2, 300, 0, C.byref(out)) == -1    # empty window
    assert lib.xkv_prefill_workspace_bytes(C.byref(s), 2, 4, 8, C.byref(out)) == -1      # window > prompt
    assert lib.xkv_prefill_workspace_bytes(C.byref(s), 2, 300, 40, C.byref(out)) == -4   # ows * G > 64
    call = lambda *a: lib.xkv_prefill_evict(C.byref(s), *a)
    ok_args = lambda **o: [o.get("l0", 0), o.get("l1", 2), o.get("q", p), o.get("k", p), o.get("v", p),
                           o.get("t", 300), o.get("tps", None), o.get("ows", 8), o.get("ps", 7),
                           o.get("bud", bud.ctypes.data), o.get("scale", 0.0), None, o.get("ws", p),
                           o.get("wsb", big), None]
    assert call(*ok_args(l1=3)) == -1
    assert call(*ok_args(q=None)) == -1
    assert call(*ok_args(k=0x2008)) == -1                                # misaligned source
    assert call(*ok_args(ps=4)) == -1                                    # even pooling width
    assert call(*ok_args(ows=0)) == -1
    assert call(*ok_args(ows=40)) == -4
    assert call(*ok_args(scale=-1.0)) == -1
    assert call(*ok_args(bud=None)) == -1
    small = np.array([50, 7, 50, 50], np.int32)                          # budget below the window
    assert call(*ok_args(bud=small.ctypes.data)) == -1
    large = np.array([50, 101, 50, 50], np.int32)                        # more than the stream holds
    assert call(*ok_args(bud=large.ctypes.data)) == -3
    assert call(*ok_args(wsb=64)) == -3
    assert call(*ok_args(ws=0x2010)) == -1                               # misaligned workspace
    short = np.array([300, 7], np.int32)                                 # a prompt shorter than the window
    assert call(*ok_args(tps=short.ctypes.data)) == -1
    long_ = np.array([301, 100], np.int32)                               # longer than the row count
    assert call(*ok_args(tps=long_.ctypes.data)) == -1
    seqs = np.array([300, 60], np.int32)                                 # budget 50 <= 60: fits, so the
    assert call(*ok_args(tps=seqs.ctypes.data, wsb=64)) == -3            # next check (workspace) is reached
    assert keep["len"].tolist() == [10, 20, 30, 100]


def test_device_allocator_and_window_importance_argument_errors():
    lib = xkv.load()
    p = 0x2000
    big = 1 << 30
    out = C.c_size_t(0)
    assert lib.xkv_allocate_device_workspace_bytes(4, 1000, C.byref(out)) == 0 and out.value > 0
    assert lib.xkv_allocate_device_workspace_bytes(0, 1000, C.byref(out)) == -1
    assert lib.xkv_allocate_device_workspace_bytes(300, 1000, C.byref(out)) == -4       # too many layers
    bud = np.zeros(4, np.int64)
    lo = np.array([10, 10, 10, 10], np.int64)
    hi = np.array([20, 20, 20, 5], np.int64)
    call = lambda *a: lib.xkv_allocate_budgets_device(*a)
    assert call(4, p, 1000, 1000, 0, 100, 0.0, None, None, None, None, p, big, None) == -1      # no output
    assert call(4, p, 1000, 999, 0, 100, 0.0, None, None, bud.ctypes.data, None, p, big, None) == -1   # stride < len
    assert call(4, p, 1000, 1000, 0, 4001, 0.0, None, None, bud.ctypes.data, None, p, big, None) == -2  # more than there is
    assert call(4, p, 1000, 1000, 0, 30, 0.0, lo.ctypes.data, None, bud.ctypes.data, None, p, big, None) == -2  # below the floors
    assert call(4, p, 1000, 1000, 0, 50, 0.0, lo.ctypes.data, hi.ctypes.data, bud.ctypes.data, None, p, big, None) == -2  # floor > cap
    assert call(4, p, 1000, 1000, 0, 100, 0.0, None, None, bud.ctypes.data, None, p, 64, None) == -3
    assert call(4, p, 1000, 1000, 0, 100, 0.0, None, None, bud.ctypes.data, None, 0x2010, big, None) == -1
    assert call(4, p, 1000, 1000, 7, 100, 0.0, None, None, bud.ctypes.data, None, p, big, None) == -1    # unknown mode
    assert call(4, p, 1000, 1000, 1, 0, 1.5, None, None, bud.ctypes.data, None, p, big, None) == -1     # target > 1
    s, keep = _fake_cache()
    wi = lambda *a: lib.xkv_window_importance(C.byref(s), *a)
    assert wi(0, 2, p, p, 300, None, 8, 7, 0.0, None, p, big, None) == -1               # no output
    assert wi(0, 2, p, p, 300, None, 8, 6, 0.0, p, p, big, None) == -1                  # even pooling width
    assert wi(0, 2, p, p, 300, None, 40, 7, 0.0, p, p, big, None) == -4
    assert wi(0, 2, p, p, 300, None, 8, 7, 0.0, p, p, 64, None) == -3
    bad = np.array([300, 3], np.int32)
    assert wi(0, 2, p, p, 300, bad.ctypes.data, 8, 7, 0.0, p, p, big, None) == -1       # prompt < window


def test_workload_generators_are_seeded_and_consistent():
    w = wl.WORKLOADS["mistral_7b_gqa_b32"]
    b1 = wl.dirichlet_budgets(w.n_layers, 4, w.context, w.total_budget, w.seed)
    b2 = wl.dirichlet_budgets(w.n_layers, 4, w.context, w.total_budget, w.seed)
    np.testing.assert_array_equal(b1, b2)
    assert w.total_budget == 157286 and np.all(b1.sum(0) == w.total_budget)
    assert b1.min() >= 64 and b1.max() <= w.context
    assert wl.WORKLOADS["llama2_7b_32k"].total_budget == 209715
    assert wl.WORKLOADS["llama3_70b_128k"].total_budget == 1572864
    off, cap, slots = wl.region_table(np.array([[8, 16], [24, 8]]), 4)
    assert off.tolist() == [0, 32, 96, 192] and slots == 224


# ---- averaged allocation lists (host only) ----
def test_average_allocations_matches_oracle():
    from oracle import xkv_oracle as orc
    r = np.random.default_rng(3)
    for trial in range(200):
        L, S = int(r.integers(1, 9)), int(r.integers(1, 6))
        lists = r.integers(0, 50, size=(S, L))
        if lists.sum() == 0:
            lists[0, 0] = 3
        use_bounds = trial % 3 == 0
        lo = r.integers(0, 10, size=L) if use_bounds else None
        hi = (lo + r.integers(0, 60, size=L)) if use_bounds else None
        N = int(r.integers(lo.sum(), hi.sum() + 1)) if use_bounds else int(r.integers(0, 400))
        got = xkv.xkv_average_allocations(lists, N, lo, hi)
        ref = orc.average_allocations(lists, N, lo, hi)
        assert np.array_equal(got, ref), (trial, lists, N, lo, hi, got, ref)
    # the lists that the allocator gives for similar tasks, averaged, still sum to the total
    curves = [wl.zipf_importance_curves(6, 300, seed=s) for s in range(4)]
    lists = np.stack([xkv.xkv_allocate_budgets(c, total_size=500)[0] for c in curves])
    avg = xkv.xkv_average_allocations(lists, 500)
    assert avg.sum() == 500 and np.all(avg >= lists.min(axis=0)) and np.all(avg <= lists.max(axis=0))


def test_average_allocations_errors():
    lib = xkv.load()
    lists = np.array([[1, 2], [3, 4]], np.int64)
    out = np.zeros(2, np.int64)
    f = lambda *a: lib.xkv_average_allocations(*a)
    assert f(2, 2, lists.ctypes.data, 10, None, None, out.ctypes.data) == 0 and out.tolist() == [4, 6]
    assert f(0, 2, lists.ctypes.data, 10, None, None, out.ctypes.data) == -1
    assert f(2, 2, None, 10, None, None, out.ctypes.data) == -1
    assert f(2, 2, lists.ctypes.data, -1, None, None, out.ctypes.data) == -1
    neg = np.array([[1, -2], [3, 4]], np.int64)
    assert f(2, 2, neg.ctypes.data, 10, None, None, out.ctypes.data) == -1
    zero = np.zeros((2, 2), np.int64)
    assert f(2, 2, zero.ctypes.data, 10, None, None, out.ctypes.data) == -1
    lo = np.array([8, 8], np.int64)
    assert f(2, 2, lists.ctypes.data, 10, lo.ctypes.data, None, out.ctypes.data) == -2
    hi = np.array([3, 3], np.int64)
    assert f(2, 2, lists.ctypes.data, 10, None, hi.ctypes.data, out.ctypes.data) == -2
