"""Host-side pieces of bench.py that need no GPU: the algorithmic byte count, the
core count rule and the oracle's worker pool of the all-cores baseline leg."""
import os

import numpy as np

import bench
import xkv_workloads as wl


def test_algorithmic_bytes_is_520_per_token_head_for_the_benchmark_geometry():
    w = wl.WORKLOADS["llama2_7b_32k"]
    lens = np.array([10, 20, 30], np.int32)
    assert bench.algorithmic_bytes(w, lens) == 60 * w.n_kv_heads * 520
    tiny = wl.WORKLOADS["tiny_f32"]                      # fp32, 64 channels: 2 * 64 * 4 + 8 as well
    assert bench.algorithmic_bytes(tiny, np.array([1], np.int32)) == tiny.n_kv_heads * 520


def test_usable_cores_follows_the_box_share(monkeypatch):
    host = len(os.sched_getaffinity(0))
    monkeypatch.setenv("OMP_NUM_THREADS", "1")
    assert bench.usable_cores() == (host, 1)
    monkeypatch.setenv("OMP_NUM_THREADS", str(10 ** 6))
    monkeypatch.delenv("MAX_JOBS", raising=False)
    assert bench.usable_cores() == (host, host)
    monkeypatch.setenv("OMP_NUM_THREADS", "not a number")
    assert bench.usable_cores() == (host, host)


def _unit(n, seed):
    r = np.random.default_rng(seed)
    bits = lambda a: (a.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)   # bf16 storage
    K, V = bits(r.standard_normal((n, 128))), bits(r.standard_normal((n, 128)))
    return (K, V, r.random(n).astype(np.float32), np.arange(n, dtype=np.int32),
            bits(r.standard_normal((1, 128))), K[0].copy(), V[0].copy(), n, n)


def test_oracle_pool_runs_every_unit_step_and_ends():
    pool = bench.OraclePool(2)
    try:
        lists = [[_unit(50, 1), _unit(70, 2)], [_unit(30, 3)]]
        wall, results = pool.run(lists, count=5, timeout=60.0)
        # worker 0 alternates its two units (51 + 71 + 51 + 71 + 51 tokens), worker 1 repeats its one
        assert [r[0] for r in results] == [51 * 3 + 71 * 2, 31 * 5]
        assert wall > 0 and all(r[1] > 0 for r in results)
        procs = [p for p, _ in pool.procs]
    finally:
        pool.close()
    assert not any(p.is_alive() for p in procs)
