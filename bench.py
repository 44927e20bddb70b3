#!/usr/bin/env python3
"""Benchmark of the XKV decode hot path on one MI355X.

A *step* is one decode step of the whole path over every layer: append the new
token, attention over the ragged cache with per-token scoring, then top-budget
eviction and compaction: xkv_decode_step, which is xkv_decode_attend_score
followed by xkv_evict_compact as one call (--two-calls times the two calls
instead).  The cache starts from the full prompt; the first warm-up
step therefore evicts context+1 -> budget in every layer (`step0_ms`), the live
tokens then move into an arena sized by the budgets (xkv_repack), and the timed
steps run in the steady state budget+1 -> budget.

Timing protocol: W untimed warm-up steps, then R repetitions of K steps, each
repetition bracketed by HIP events on the launch stream; `ms_per_step` and
`value` are the median repetition, the spread is reported beside it.  Giving the
prompt-sized arena back makes the driver clear the freed memory in the
background, which slows everything that runs meanwhile by about 5 %; the
benchmark times a few steps inside that window (`ms_per_step_during_vram_release`)
and then waits for it to pass before the timed repetitions.

Prints ONE JSON line: decode attend+evict layer-steps per second (layers x
steps / elapsed) of the metric's workload, the HBM roofline of the dominant
kernel, the CPU oracle's rate on a bounded sample of the same work (one thread,
and one process per host core), and `other_workloads`: the same measurement,
shortened, for the other benchmark configurations.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
VRAM_CLEAR_GBS = 20.0          # pessimistic rate at which freed device memory is cleared (measured: about 30)
ALL_WORKLOADS = ("tiny_f32", "llama2_7b_4k", "llama2_7b_32k", "mistral_7b_gqa_b32", "llama3_70b_128k")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed decode steps per repetition (default: the workload's run minus warm-up)")
    ap.add_argument("--warmup", type=int, default=1, help="untimed steps; the first one is the prompt-sized eviction")
    ap.add_argument("--reps", type=int, default=5, help="timed repetitions of --steps steps; the median is reported")
    ap.add_argument("--workload", default="llama2_7b_32k")
    ap.add_argument("--others", default="all",
                    help="'all', 'none' or a comma-separated list: the other workloads measured (shortened) into other_workloads")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="CPU time budget of each leg of the oracle baseline (0 = skip)")
    ap.add_argument("--no-roofline-pass", action="store_true")
    ap.add_argument("--keep-prompt-arena", action="store_true",
                    help="stay in the prompt-sized arena after the first eviction instead of moving to one sized by the budgets")
    ap.add_argument("--evict-every", type=int, default=1,
                    help="decode steps between evictions (1 = every step; 8 = once per observation window)")
    ap.add_argument("--n-protect", type=int, default=0, help="most recent tokens that are never evicted")
    ap.add_argument("--pool-size", type=int, default=1, help="pooling width of the eviction keys (odd)")
    ap.add_argument("--attend-path", type=int, default=0,
                    help="0 library's choice, 1 streaming + finalize kernels, 2 fused cooperative launch")
    ap.add_argument("--no-graph", action="store_true", help="skip the graph-replay figure")
    ap.add_argument("--no-prefill", action="store_true", help="skip the prefill-phase eviction leg")
    ap.add_argument("--two-calls", action="store_true",
                    help="a step is xkv_decode_attend_score then xkv_evict_compact instead of xkv_decode_step")
    ap.add_argument("--no-settle", action="store_true", help="do not wait for the freed prompt arena to be cleared")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain device copy of 1 GiB x 10 (reference point for HBM byte counters)")
    return ap.parse_args()


def note(msg):
    """Progress line on stderr (the result line on stdout stays the only one there)."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def make_budgets(xkv, wl, w):
    """int32 [L, B] per the workload's rule; also returns allocator timings."""
    import numpy as np
    info = {}
    if w.budget_rule == "fixed":
        bud = np.repeat(np.asarray(w.fixed_budgets, np.int32)[:, None], w.batch, axis=1)
    elif w.budget_rule == "dirichlet":
        bud = wl.dirichlet_budgets(w.n_layers, w.batch, w.context, w.total_budget, w.seed)
    else:
        curves = wl.zipf_importance_curves(w.n_layers, w.context, w.seed)
        floor = [w.min_budget] * w.n_layers if w.min_budget else None
        t0 = time.perf_counter()
        b1, ravg = xkv.xkv_allocate_budgets(curves, total_size=w.total_budget, min_budget=floor)
        info = {"lib_ms": (time.perf_counter() - t0) * 1e3, "r_avg": ravg, "curves": curves, "floor": floor}
        bud = np.repeat(b1.astype(np.int32)[:, None], w.batch, axis=1)
    return np.ascontiguousarray(bud, dtype=np.int32), info


def repack(cache, budgets, slack=1, stream=None):
    """Moves the live tokens into a cache whose streams have room for budget +
    slack tokens only (rounded up to 8 slots): the memory the method saves is
    actually released, and the steady state runs in the small arena."""
    import numpy as np
    caps = ((budgets.astype(np.int64) + slack + 7) // 8 * 8).astype(np.int32)
    return cache.resized(caps, stream=stream)


def algorithmic_bytes(w, lens_after_append):
    """K and V rows read once plus the fp32 score read and written, per live
    token per KV head: (2*d*e + 8) bytes."""
    per_token = 2 * w.head_dim * w.elem_bytes + 8
    return int(lens_after_append.astype("int64").sum()) * w.n_kv_heads * per_token


# ---------------------------------------------------------------------------
# CPU baseline: the oracle as it stands, one thread and one process per core
# ---------------------------------------------------------------------------
def _oracle_unit_step(unit):
    """One steady-state step of one (layer, sequence, KV head) unit on the oracle:
    append, attention + scoring, eviction.  Returns the tokens it covered."""
    from oracle import xkv_oracle as orc
    K, V, sc, ps, qq, kk, vv, pos_new, budget = unit
    u = orc.OracleUnit(K, V, sc, ps)
    u.append(kk, vv, pos_new)
    u.attend(qq)
    u.evict(budget)
    return K.shape[0] + 1


def _oracle_worker(conn):
    """Child process of the all-cores leg: receives its units, waits for "go", runs
    them on one thread and reports (tokens, seconds); "quit" ends it."""
    # one thread per process: set before NumPy loads its BLAS, and again on what is loaded
    for var in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS"):
        os.environ[var] = "1"
    from oracle import xkv_oracle  # noqa: F401
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(limits=1)
    except Exception:                                   # pragma: no cover
        pass
    units, count = [], 0
    while True:
        try:
            msg = conn.recv()
        except EOFError:
            return
        if msg == "quit":
            return
        if msg == "go":
            t0 = time.perf_counter()
            tokens = sum(_oracle_unit_step(units[i % len(units)]) for i in range(count))
            conn.send((tokens, time.perf_counter() - t0))
        else:
            units, count = msg                          # distinct units, and how many unit-steps to run over them in turn
            conn.send("ready")


class OraclePool:
    """Worker processes of the all-cores oracle leg.  They are started before this
    process touches the GPU (a process that has initialised the GPU must not start
    other programs) and idle until the leg runs; they never use the GPU."""

    def __init__(self, n):
        import multiprocessing as mp
        ctx = mp.get_context("fork")
        self.procs = []
        for _ in range(n):
            parent, child = ctx.Pipe()
            p = ctx.Process(target=_oracle_worker, args=(child,), daemon=True)
            p.start()
            child.close()
            self.procs.append((p, parent))

    def run(self, unit_lists, count, timeout=90.0):
        """Hands list i to worker i, which runs `count` unit-steps over it in turn; all start at
        once -> (wall seconds, [(tokens, seconds)])."""
        for (p, conn), units in zip(self.procs, unit_lists):
            if not p.is_alive():
                raise RuntimeError(f"oracle worker {p.pid} is gone (exit code {p.exitcode})")
            conn.send((units, count))
        for _, conn in self.procs:
            if not conn.poll(timeout) or conn.recv() != "ready":
                raise RuntimeError("an oracle worker did not report ready")
        t0 = time.perf_counter()
        for _, conn in self.procs:
            conn.send("go")
        results = []
        for _, conn in self.procs:
            if not conn.poll(timeout):
                raise RuntimeError("an oracle worker did not finish")
            results.append(conn.recv())
        return time.perf_counter() - t0, results

    def close(self):
        for p, conn in self.procs:
            try:
                conn.send("quit")
            except Exception:
                pass
        for p, _ in self.procs:
            p.join(timeout=5)
            if p.is_alive():
                p.terminate()
        self.procs = []


def usable_cores():
    """Host cores this process may run on, and how many the all-cores leg uses
    (the box's share of the host can be smaller than its affinity mask: the
    thread-count variables it exports say so)."""
    host = len(os.sched_getaffinity(0))
    share = host
    for var in ("OMP_NUM_THREADS", "MAX_JOBS"):
        try:
            share = min(share, int(os.environ[var]))
        except (KeyError, ValueError):
            pass
    return host, max(share, 1)


def cpu_baseline(w, wl, cache, budgets, inputs, t, seconds, pool):
    """The oracle on a seeded sample of steady-state unit-steps taken from the
    cache as it stands: (a) one thread in this process for `seconds`; (b) one
    process per usable core over independent units, sized from (a) to take about
    as long.  Rates are extrapolated by token count to the whole layer-step."""
    import numpy as np
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)
    except Exception:                                   # pragma: no cover
        limiter = None
    q_all, kn_all, vn_all, gen_steps = inputs
    G = w.group
    units = [(l, b, h) for l in range(w.n_layers) for b in range(w.batch) for h in range(w.n_kv_heads)]
    order = np.random.default_rng(w.seed).permutation(len(units))
    cursor = [0]

    def next_unit():
        k = cursor[0]
        cursor[0] += 1
        passes, idx = divmod(k, len(units))
        l, b, h = units[order[idx]]
        i = (t + passes) % gen_steps
        n = cache.length(l, b)
        s0 = cache.stream_slot(l, b, h)
        return (wl.to_numpy_storage(cache.k[s0:s0 + n]), wl.to_numpy_storage(cache.v[s0:s0 + n]),
                cache.score[s0:s0 + n].cpu().numpy(), cache.pos[s0:s0 + n].cpu().numpy(),
                wl.to_numpy_storage(q_all[i][l, b, h * G:(h + 1) * G]), wl.to_numpy_storage(kn_all[i][l, b, h]),
                wl.to_numpy_storage(vn_all[i][l, b, h]), w.context + t + passes, int(budgets[l, b]))

    mean_tokens_per_layer_step = float((budgets.astype("int64") + 1).sum()) * w.n_kv_heads / w.n_layers

    # (a) one thread
    spent, done, tokens = 0.0, 0, 0
    while spent < seconds:
        u = next_unit()
        t0 = time.perf_counter()
        tokens += _oracle_unit_step(u)
        spent += time.perf_counter() - t0
        done += 1
    rate1 = tokens / spent
    if limiter is not None and hasattr(limiter, "restore_original_limits"):
        limiter.restore_original_limits()
    host, cores = usable_cores()
    single = {"value": rate1 / mean_tokens_per_layer_step, "unit": "layer-steps/s", "cores": 1, "kind": "oracle",
              "host_cores": host,
              "sample": f"{done} (layer, sequence, KV-head) unit-steps of the {len(units)} per step, "
                        f"{spent:.1f} s of NumPy float64 on one thread, extrapolated by token count "
                        f"({w.batch * w.n_kv_heads} units per layer-step)"}

    # (b) one process per core over independent units
    if pool is None:
        return single
    cores = len(pool.procs)
    note(f"one thread: {done} unit-steps in {spent:.1f} s; now {cores} processes")
    per_proc = max(1, int(round(done * min(seconds, spent) / spent)))
    try:
        distinct = min(per_proc, 24)                     # bounded host memory: a unit holds its K and V rows
        wall, results = pool.run([[next_unit() for _ in range(distinct)] for _ in range(cores)], per_proc)
        tok_all = sum(r[0] for r in results)
        single["all_cores"] = {
            "value": (tok_all / wall) / mean_tokens_per_layer_step, "unit": "layer-steps/s", "cores": cores,
            "kind": "oracle",
            "sample": f"{cores} processes x {per_proc} unit-steps each over {distinct} distinct units of its own, one NumPy thread per process, "
                      f"{wall:.1f} s wall (slowest process {max(r[1] for r in results):.1f} s), extrapolated by token count"}
    except Exception as e:                              # pragma: no cover
        single["all_cores"] = {"error": repr(e), "cores": cores}
    return single


# ---------------------------------------------------------------------------
# one workload
# ---------------------------------------------------------------------------
def warm_kernels(xkv, wl, w, torch, np, stream):
    """One tiny call of every kernel the run will use, on a scratch cache of the
    workload's head geometry: the first launch of a kernel loads its code object,
    which would otherwise be counted into the first step."""
    lens = np.full((2, w.batch), 17, np.int32)
    lens[0, 0] = 300
    c = xkv.XkvCache(2, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, lens + 600)
    c.len[:] = lens.reshape(-1)
    tdt = w.torch_dtype()
    q = torch.zeros((2, w.batch, w.n_q_heads, w.head_dim), dtype=tdt, device="cuda")
    kn = torch.zeros((2, w.batch, w.n_kv_heads, w.head_dim), dtype=tdt, device="cuda")
    o = torch.empty((2, w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    ws = torch.empty(xkv.xkv_workspace_bytes(c, 2), dtype=torch.uint8, device="cuda")
    pn = np.zeros(w.batch, np.int32)
    for bud in (200, 10 ** 6):
        xkv.xkv_decode_attend_score(c, 0, 2, q, kn, kn, pn, o, ws, stream=stream)
        xkv.xkv_evict_compact(c, 0, 2, np.full((2, w.batch), bud, np.int32), ws, stream=stream)
    xkv.xkv_decode_step(c, 0, 2, q, kn, kn, pn, o, c.len.reshape(2, w.batch).copy(), ws, stream=stream)   # one in, one out
    c2 = c.resized(lens + 8, stream=stream)
    torch.cuda.synchronize()
    del c, c2, ws


def run_workload(xkv, wl, w, args, K, W, R, full, pool=None):
    """Measures one workload.  full: also the graph replay, the read ceiling, the
    prefill leg, the CPU baseline and the allocator timings (the metric's workload)."""
    import numpy as np
    import torch

    L, B = w.n_layers, w.batch
    every = max(args.evict_every, 1) if full else 1
    pool_size = args.pool_size if full else 1
    n_protect = args.n_protect if full else 0
    if every > 1:
        W = max(W, every)                     # the warm-up ends with the first (prompt-sized) eviction
    W = max(W, 1)
    stream = torch.cuda.current_stream()

    note(f"workload {w.name}: budgets")
    budgets, alloc = make_budgets(xkv, wl, w)
    if n_protect > 0:
        budgets = np.maximum(budgets, n_protect).astype(np.int32)
    warm_kernels(xkv, wl, w, torch, np, stream)
    caps = np.full((L, B), wl.round_up(w.context + every, 8), dtype=np.int32)
    cache = xkv.XkvCache(L, B, w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, caps)
    wl.fill_prompt_cache(w, cache.k, cache.v, cache.score, cache.pos, cache.region_off, cache.cap)
    cache.len[:] = w.context
    gen_steps = min(W + (R + 2) * K + 8, 128)
    q, kn, vn, _ = wl.decode_inputs(w, steps=gen_steps, device="cuda")
    out = torch.empty((L, B, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    ws = torch.empty(xkv.xkv_workspace_bytes(cache, L), dtype=torch.uint8, device="cuda")
    pos_step = np.zeros(B, np.int32)
    alg_bytes = [0]
    state = {"cache": cache, "ws": ws, "t": 0}

    def step():
        t = state["t"]
        i = t % gen_steps
        c = state["cache"]
        pos_step[:] = w.context + t
        alg_bytes[0] += algorithmic_bytes(w, c.len + 1)
        if (t + 1) % every != 0:
            xkv.xkv_decode_attend_score(c, 0, L, q[i], kn[i], vn[i], pos_step, out, state["ws"], stream=stream)
        elif args.two_calls:
            xkv.xkv_decode_attend_score(c, 0, L, q[i], kn[i], vn[i], pos_step, out, state["ws"], stream=stream)
            xkv.xkv_evict_compact(c, 0, L, budgets, state["ws"], pool_size=pool_size, n_protect=n_protect,
                                  stream=stream)
        else:
            xkv.xkv_decode_step(c, 0, L, q[i], kn[i], vn[i], pos_step, out, budgets, state["ws"],
                                pool_size=pool_size, n_protect=n_protect, stream=stream)
        state["t"] = t + 1

    def timed(n):
        """n steps between two events on the launch stream -> ms per step."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(n):
            step()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    note("prompt cache filled; first steps (the first eviction cuts every layer to its budget)")
    torch.cuda.synchronize()
    step0_ms, repack_ms, release_ms, settle_s = None, None, None, 0.0
    prompt_arena_bytes = int(2 * cache.arena_slots * w.head_dim * w.elem_bytes)
    for _ in range(every):                    # up to and including the first eviction
        t0 = time.perf_counter()
        ms = timed(1)
        if step0_ms is None:
            step0_ms = ms
            step0_host_ms = (time.perf_counter() - t0) * 1e3
    if not args.keep_prompt_arena:
        # the prompt-sized arena has done its job: continue in one sized by the budgets
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        packed = repack(cache, budgets, slack=every, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        repack_ms = e0.elapsed_time(e1)
        freed = (cache.k.numel() * cache.k.element_size() * 2 + cache.score.numel() * 8 + ws.numel())
        del ws, cache
        state["cache"] = state["ws"] = None
        torch.cuda.empty_cache()
        cache = packed
        ws = torch.empty(xkv.xkv_workspace_bytes(cache, L), dtype=torch.uint8, device="cuda")
        state["cache"], state["ws"] = cache, ws
        if every == 1:
            release_ms = timed(min(K, 8))     # inside the window in which the freed arena is being cleared
        if not args.no_settle:
            settle_s = freed / (VRAM_CLEAR_GBS * 1e9) + 0.5
            note(f"waiting {settle_s:.1f} s for the driver to clear the {freed / 1e9:.1f} GB just freed")
            time.sleep(settle_s)
    while state["t"] < W:
        step()
    torch.cuda.synchronize()

    note(f"timing {R} x {K} steps")
    reps, rep_bytes = [], []
    host0 = time.perf_counter()
    for _ in range(R):
        alg_bytes[0] = 0
        reps.append(timed(K))
        rep_bytes.append(alg_bytes[0] / K)
    host_ms_per_step = (time.perf_counter() - host0) * 1e3 / (R * K)
    ms_per_step = statistics.median(reps)
    alg_step = statistics.median(rep_bytes)
    step_gbs = alg_step / (ms_per_step * 1e-3) / 1e9
    steady = bool(np.all(cache.len.reshape(L, B) < budgets + every))

    roofline = None
    if not args.no_roofline_pass:
        note("roofline pass")
        alg_bytes[0] = 0
        xkv.xkv_profile_enable(True)
        for _ in range(K):
            step()
        torch.cuda.synchronize()
        alg_bytes_step = alg_bytes[0] / K
        launches, total_ms = xkv.xkv_profile_read(0)
        sel_launches, sel_ms = xkv.xkv_profile_read(1)
        se_launches, se_ms = xkv.xkv_profile_read(3)
        xkv.xkv_profile_enable(False)
        launches_per_step = launches / K
        bytes_per_launch = alg_bytes_step / launches_per_step
        achieved = bytes_per_launch / (total_ms / launches * 1e-3) / 1e9
        traffic, traffic_source = None, None
        tname = f"decode_kernels_{w.name}_hbm_traffic.txt"
        tfile = os.path.join(ROOT, "profiles", tname)
        if os.path.exists(tfile):
            for line in open(tfile):
                if line.startswith("traffic_bytes_per_launch:"):
                    traffic = float(line.split(":")[1])
                    traffic_source = (f"profiles/{tname}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                      f"kernel on this workload, collected separately and committed; not measured in this run")
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                    "kernel": ("attend_strip" if w.group <= 2 else "attend_gqa") +
                              " (K/V streaming kernel of xkv_decode_attend_score)",
                    "avg_launch_ms": total_ms / launches,
                    "launches_per_step": launches_per_step, "algorithmic_bytes_per_launch": bytes_per_launch,
                    "evict_select_avg_ms": (sel_ms / sel_launches) if sel_launches else None,
                    "score_and_evict_avg_ms": (se_ms / se_launches) if se_launches else None}

    res = {
        "workload": w.name, "ms_per_step": ms_per_step, "layer_steps_per_s": L / (ms_per_step * 1e-3),
        "steps": K, "reps": R, "ms_per_step_reps": reps,
        "ms_per_step_spread": (max(reps) - min(reps)) / ms_per_step,
        "host_clock_ms_per_step": host_ms_per_step,
        "algorithmic_bytes_per_step": alg_step, "step_hbm_gbs": step_gbs, "step_hbm_frac": step_gbs / HBM_PEAK_GBS,
        "kernel": roofline["kernel"].split(" ")[0] if roofline else None,
        "kernel_frac": roofline["frac"] if roofline else None,
        "kernel_avg_launch_ms": roofline["avg_launch_ms"] if roofline else None,
        "step0_ms": step0_ms, "step0_host_clock_ms": step0_host_ms, "repack_ms": repack_ms,
        "ms_per_step_during_vram_release": release_ms, "settle_s": settle_s,
        "prompt_arena_bytes": prompt_arena_bytes,
        "kv_arena_bytes": int(2 * cache.arena_slots * w.head_dim * w.elem_bytes),
        "steady_state": steady,
    }
    # the whole run as the workload defines it: the prompt-sized first step, the move, then steady steps
    run_ms = step0_ms + (repack_ms or 0.0) + (w.decode_steps - 1) * ms_per_step
    res["whole_run"] = {"decode_steps": w.decode_steps, "ms": run_ms,
                        "layer_steps_per_s": L * w.decode_steps / (run_ms * 1e-3),
                        "note": "step0_ms + repack_ms + (decode_steps - 1) x ms_per_step, all measured in this run"}
    if w.name == "tiny_f32":
        res["note"] = "cache-resident (1.7 MB): its GB/s is no statement about HBM"
    elif w.name == "llama2_7b_4k":
        res["note"] = "0.86 GB retained: partly resident in the 256 MB last-level cache"
    if not full:
        del cache, ws, q, kn, vn, out
        state.clear()
        torch.cuda.empty_cache()
        return res, None

    extra = {"roofline": roofline, "budgets": budgets}
    # The same step captured once in a HIP graph and replayed (extra figure, not `value`: every
    # replay appends the captured step's token and position again).
    graph_ms = None
    if every == 1 and not args.no_graph:
        note("graph replay")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        gr = torch.cuda.CUDAGraph()
        i = state["t"] % gen_steps
        pos_step[:] = w.context + state["t"]
        with torch.cuda.stream(side):
            with torch.cuda.graph(gr, stream=side):
                if args.two_calls:
                    xkv.xkv_decode_attend_score(cache, 0, L, q[i], kn[i], vn[i], pos_step, out, ws, stream=side)
                    xkv.xkv_evict_compact(cache, 0, L, budgets, ws, pool_size=pool_size, n_protect=n_protect,
                                          stream=side)
                else:
                    xkv.xkv_decode_step(cache, 0, L, q[i], kn[i], vn[i], pos_step, out, budgets, ws,
                                        pool_size=pool_size, n_protect=n_protect, stream=side)
        torch.cuda.current_stream().wait_stream(side)
        gr.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            gr.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / K * 1e3
        del gr
    extra["graph_ms"] = graph_ms

    # What a read-only kernel of the same shape reaches on this machine (context for the roofline fraction).
    ceiling = None
    if not args.no_roofline_pass:
        buf = cache.k
        per_wg = 128 * 1024
        nbytes = buf.numel() * buf.element_size() // per_wg * per_wg
        sink = torch.empty((nbytes // per_wg) * 1024, dtype=torch.float32, device="cuda")
        ceiling = {"bytes_per_launch": nbytes}
        # loads: non-temporal or ordinary; then non-temporal loads with 1.5 KB (a strip record) or 4 KB
        # stored per 128 KiB read, under the three store policies
        cases = [("non_temporal_GBs", True, 0, 2), ("ordinary_loads_GBs", False, 0, 2)]
        for fl, label in ((386, "1544B"), (1024, "4096B")):
            for pol, pname in ((0, "ordinary"), (1, "non_temporal"), (2, "system_scope")):
                cases.append((f"non_temporal_with_{label}_{pname}_store_per_128KiB_GBs", True, fl, pol))
        for tag, nt, st, pol in cases:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            xkv.xkv_probe_stream_read(buf, nt, st, sink, stream=stream, store_policy=pol)
            e0.record(stream)
            for _ in range(20):
                xkv.xkv_probe_stream_read(buf, nt, st, sink, stream=stream, store_policy=pol)
            e1.record(stream)
            torch.cuda.synchronize()
            ceiling[tag] = nbytes * 20 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del sink
    extra["ceiling"] = ceiling

    extra["prefill"] = None if args.no_prefill else prefill_leg(xkv, wl, w, budgets, torch, np, stream)

    cpu = None
    if args.cpu_seconds > 0:
        note("oracle on the host cores")
        cpu = cpu_baseline(w, wl, cache, budgets, (q, kn, vn, gen_steps), state["t"], args.cpu_seconds, pool)
    extra["cpu"] = cpu

    allocator = None
    if alloc:
        note("allocator timings")
        from oracle import xkv_oracle as orc
        t0 = time.perf_counter()
        ref, _ = orc.allocate_budgets(alloc["curves"], total_size=w.total_budget, min_budget=alloc["floor"])
        oracle_ms = (time.perf_counter() - t0) * 1e3
        # the same curves, already on the device (where the mini-prefill leaves them)
        dev_curves = torch.from_numpy(np.stack(alloc["curves"])).cuda()
        aws = torch.empty(xkv.xkv_allocate_device_workspace_bytes(L, w.context), dtype=torch.uint8, device="cuda")
        dev_ms, dev_bud = None, None
        for _ in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            dev_bud, _ = xkv.xkv_allocate_budgets_device(dev_curves, L, w.context, w.context, w.total_budget, aws,
                                                         min_budget=alloc["floor"])
            dev_ms = (time.perf_counter() - t0) * 1e3
        allocator = {"xkv_allocate_budgets_ms": alloc["lib_ms"], "oracle_ms": oracle_ms,
                     "xkv_allocate_budgets_device_ms": dev_ms,
                     "identical": bool(np.array_equal(ref, budgets[:, 0])),
                     "device_identical": bool(np.array_equal(dev_bud, ref)), "r_avg": alloc["r_avg"]}
        del dev_curves, aws
    extra["allocator"] = allocator
    del cache, ws, q, kn, vn, out
    state.clear()
    torch.cuda.empty_cache()
    return res, extra


def prefill_leg(xkv, wl, w, budgets, torch, np, stream, layers_per_call=(1, 4)):
    """Prefill-phase eviction (Alg. 2 as written, ows = 8, ps = 7) of the whole
    model into a budget-sized cache: `layers_per_call` dense layers of the prompt
    per call, as a prefill produces them.  The same dense layers are the source
    for every call; the budgets differ per layer."""
    note("prefill-phase eviction leg")
    L, B = w.n_layers, w.batch
    ows, ps = 8, 7
    bud_p = np.maximum(budgets, ows)
    caps_p = ((np.minimum(bud_p, w.context).astype(np.int64) + 7) // 8 * 8).astype(np.int32)
    dst = xkv.XkvCache(L, B, w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, caps_p)
    row = w.head_dim * w.elem_bytes
    kept = np.minimum(bud_p, w.context).astype(np.int64)
    # K of the prompt read once, kept K and V rows read and written, score and pos written
    pre_bytes = int(L * B * w.n_kv_heads * w.context * row + kept.sum() * w.n_kv_heads * (4 * row + 8))
    k_pass_bytes = B * w.n_kv_heads * w.context * row
    out = None
    for lpc in layers_per_call:
        if L % lpc:
            continue
        ws_p = torch.empty(xkv.xkv_prefill_workspace_bytes(dst, lpc, w.context, ows), dtype=torch.uint8, device="cuda")
        parts = [wl.dense_prompt_layer(w, i, ows, device="cuda") for i in range(lpc)]
        q_win = torch.cat([p[0] for p in parts]); k_src = torch.cat([p[1] for p in parts]); v_src = torch.cat([p[2] for p in parts])
        del parts
        xkv.xkv_prefill_evict(dst, 0, lpc, q_win, k_src, v_src, w.context, ows, bud_p[0:lpc], ws_p, pool_size=ps,
                              stream=stream)                                 # warm-up
        torch.cuda.synchronize()
        def timed(call):
            reps = []
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for l in range(0, L, lpc):
                    call(l)
                e1.record(stream)
                torch.cuda.synchronize()
                reps.append(e0.elapsed_time(e1) * 1e-3)
            if xkv.xkv_fused_status():
                raise RuntimeError("a wait of the one-launch selection gave up during the prefill leg")
            return statistics.median(reps)

        xkv.xkv_profile_enable(True)
        dt = timed(lambda l: xkv.xkv_prefill_evict(dst, l, l + lpc, q_win, k_src, v_src, w.context, ows,
                                                   bud_p[l:l + lpc], ws_p, pool_size=ps, stream=stream))
        n_stats, ms_stats = xkv.xkv_profile_read(2)
        xkv.xkv_profile_enable(False)
        # The same with the window rows' normalisers given, as an attention forward pass over the prompt
        # leaves them (computed here with torch, outside the timed region): K is read once.
        lse = window_row_lse_torch(torch, q_win, k_src, w.n_q_heads // w.n_kv_heads)
        xkv.xkv_prefill_evict_lse(dst, 0, lpc, q_win, k_src, v_src, w.context, ows, bud_p[0:lpc], lse, ws_p,
                                  pool_size=ps, stream=stream)
        torch.cuda.synchronize()
        dt_lse = timed(lambda l: xkv.xkv_prefill_evict_lse(dst, l, l + lpc, q_win, k_src, v_src, w.context, ows,
                                                           bud_p[l:l + lpc], lse, ws_p, pool_size=ps, stream=stream))
        del lse
        leg = {"layers_per_call": lpc, "ms_per_layer": dt / L * 1e3, "layers_per_s": L / dt,
               "hbm_gbs": pre_bytes / dt / 1e9, "hbm_frac": pre_bytes / dt / 1e9 / HBM_PEAK_GBS,
               "first_k_pass_avg_ms": ms_stats / n_stats if n_stats else None,
               "first_k_pass_hbm_frac": (lpc * k_pass_bytes / (ms_stats / n_stats * 1e-3) / 1e9 / HBM_PEAK_GBS)
               if n_stats else None,
               "with_given_row_normalisers": {"ms_per_layer": dt_lse / L * 1e3,
                                              "hbm_frac": pre_bytes / dt_lse / 1e9 / HBM_PEAK_GBS}}
        if out is None:
            out = {"ows": ows, "pool_size": ps, "algorithmic_bytes_per_layer": pre_bytes / L,
                   "note": "the same dense layers are the source for every call; budgets differ per layer; "
                           "median of 3 passes over the whole model, HIP events", "by_layers_per_call": []}
        out["by_layers_per_call"].append(leg)
        del ws_p, q_win, k_src, v_src
        torch.cuda.empty_cache()
    best = max(out["by_layers_per_call"], key=lambda x: x["hbm_frac"])
    out.update({k: best[k] for k in ("layers_per_call", "ms_per_layer", "layers_per_s", "hbm_gbs", "hbm_frac")})
    del dst
    return out


def window_row_lse_torch(torch, q_win, k_src, group):
    """ln of the softmax row sums of the window rows, [layers, B, Hq, ows] fp32, with torch ops: stands in
    for what the model's attention forward pass over the prompt hands over (input preparation, untimed)."""
    nl, B, Hq, ows, d = q_win.shape
    t = k_src.shape[3]
    out = torch.empty((nl, B, Hq, ows), dtype=torch.float32, device=q_win.device)
    col = torch.arange(t, device=q_win.device)
    seen = col[None, :] <= (t - ows + torch.arange(ows, device=q_win.device))[:, None]          # [ows, t]
    for l in range(nl):
        for b in range(B):
            q = q_win[l, b].float().reshape(Hq // group, group * ows, d)
            logits = torch.bmm(q, k_src[l, b].float().transpose(1, 2)) / math.sqrt(d)          # [Hkv, G ows, t]
            logits = logits.reshape(Hq, ows, t).masked_fill(~seen[None], float("-inf"))
            out[l, b] = torch.logsumexp(logits, dim=-1)
    return out


def gpu_unique_id():
    """Identity of the GPU the numbers come from (step times differ between boards)."""
    try:
        return open("/sys/class/drm/card0/device/unique_id").read().strip()
    except OSError:
        return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    # The oracle's worker processes start now, before anything here touches the GPU.
    pool = None
    if args.cpu_seconds > 0 and not args.calibrate_copy:
        pool = OraclePool(usable_cores()[1])
    import numpy as np
    import torch

    import paper_2412_05896_amd as xkv
    import xkv_workloads as wl

    xkv.load()
    xkv.xkv_configure(xkv.XKV_CFG_ATTEND_PATH, args.attend_path)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 10
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4,
                          "copies": 10, "ms_per_copy": dt * 1e3, "GBps_read_plus_write": 2 * src.numel() * 4 / dt / 1e9}))
        return
    w = wl.WORKLOADS[args.workload]
    W = max(args.warmup, 1)
    K = args.steps if args.steps is not None else max(w.decode_steps - W, 1)
    R = max(args.reps, 1)
    host_cores, _ = usable_cores()

    res, extra = run_workload(xkv, wl, w, args, K, W, R, full=True, pool=pool)
    if pool is not None:
        pool.close()

    others = []
    if args.others != "none":
        names = [n for n in ALL_WORKLOADS if n != w.name] if args.others == "all" else \
            [n for n in args.others.split(",") if n]
        for name in names:
            ow = wl.WORKLOADS[name]
            ko = max(1, min(K, ow.decode_steps - 1, 20))
            try:
                r, _ = run_workload(xkv, wl, ow, args, ko, min(W, 3), min(R, 5), full=False)
            except Exception as e:                      # the main figure must survive a failure here
                r = {"workload": name, "error": repr(e)}
                torch.cuda.empty_cache()
            others.append(r)

    budgets = extra["budgets"]
    line = {
        "metric": "decode attend+evict layer-steps/sec; achieved HBM GB/s vs MI355X peak",
        "value": res["layer_steps_per_s"], "unit": "layer-steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "layers": w.n_layers, "q_heads": w.n_q_heads, "kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "batch": w.batch, "context": w.context,
                   "total_budget": int(budgets[:, 0].sum()), "budget_frac": w.budget_frac,
                   "budget_min": int(budgets.min()), "budget_max": int(budgets.max()),
                   "schedule": "every step, every layer: append, attend+score" +
                               (", evict to budget" if args.evict_every <= 1 else f"; every {args.evict_every} steps: evict to budget"),
                   "pool_size": args.pool_size, "n_protect": args.n_protect, "attend_path": args.attend_path,
                   "arena": "prompt-sized" if args.keep_prompt_arena else "budget-sized after the first eviction",
                   "kv_arena_bytes": res["kv_arena_bytes"], "steady_state": res["steady_state"]},
        "timing": "median of `reps` repetitions of `steps` steps, each between HIP events on the launch stream",
        "step_call": "xkv_decode_attend_score + xkv_evict_compact" if args.two_calls else "xkv_decode_step",
        "reps": res["reps"], "ms_per_step_reps": res["ms_per_step_reps"], "ms_per_step_spread": res["ms_per_step_spread"],
        "host_clock_ms_per_step": res["host_clock_ms_per_step"],
        "step0_ms": res["step0_ms"], "step0_host_clock_ms": res["step0_host_clock_ms"], "repack_ms": res["repack_ms"],
        "ms_per_step_during_vram_release": res["ms_per_step_during_vram_release"], "settle_s": res["settle_s"],
        "whole_run": res["whole_run"], "host_cores": host_cores, "gpu_unique_id": gpu_unique_id(),
        "graph_replay_ms_per_step": extra["graph_ms"],
        "algorithmic_bytes_per_step": res["algorithmic_bytes_per_step"],
        "step_hbm_gbs": res["step_hbm_gbs"], "step_hbm_frac": res["step_hbm_frac"],
        "roofline": extra["roofline"], "stream_read_ceiling": extra["ceiling"], "prefill_evict": extra["prefill"],
        "cpu_baseline": extra["cpu"], "allocator": extra["allocator"], "other_workloads": others,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
