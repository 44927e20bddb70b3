#!/usr/bin/env python3
"""Benchmark of the XKV decode hot path on one MI355X.

A *step* is one decode step of the whole path over every layer: append the new
token, attention over the ragged cache with per-token scoring
(xkv_decode_attend_score), then top-budget eviction and compaction
(xkv_evict_compact).  The cache starts from the full prompt; the first warm-up
step therefore evicts context+1 -> budget in every layer (reported as `step0_ms`)
and the timed steps run in the steady state budget+1 -> budget.

Prints ONE JSON line: decode attend+evict layer-steps per second (layers x
steps / elapsed), the HBM roofline of the dominant kernel and the CPU oracle's
rate on a bounded sample of the same work.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed decode steps (default: the workload's run minus warm-up)")
    ap.add_argument("--warmup", type=int, default=1, help="untimed steps; the first one is the prompt-sized eviction")
    ap.add_argument("--workload", default="llama2_7b_32k")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="CPU time budget of the oracle baseline (0 = skip)")
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


def repack(cache, budgets, slack=1):
    """Moves the live tokens into a cache whose streams have room for budget +
    slack tokens only (rounded up to 8 slots): the memory the method saves is
    actually released, and the steady state runs in the small arena."""
    import numpy as np
    caps = ((budgets.astype(np.int64) + slack + 7) // 8 * 8).astype(np.int32)
    return cache.resized(caps)


def algorithmic_bytes(w, lens_after_append):
    """K and V rows read once plus the fp32 score read and written, per live
    token per KV head: (2*d*e + 8) bytes."""
    per_token = 2 * w.head_dim * w.elem_bytes + 8
    return int(lens_after_append.astype("int64").sum()) * w.n_kv_heads * per_token


def cpu_baseline(w, wl, cache, budgets, inputs, t, seconds):
    """The oracle, as it stands, on a seeded sample of units of steady-state steps
    (append + attention/scoring + eviction), one thread.  Every unit is taken from
    the cache as it stands; when all units of a step have been done before the time
    is up, the next pass uses the next step's queries and new tokens."""
    import numpy as np
    from oracle import xkv_oracle as orc
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)
    except Exception:                                   # pragma: no cover
        limiter = None
    q_all, kn_all, vn_all, gen_steps = inputs
    G = w.group
    units = [(l, b, h) for l in range(w.n_layers) for b in range(w.batch) for h in range(w.n_kv_heads)]
    order = np.random.default_rng(w.seed).permutation(len(units))
    spent, done, tokens, passes = 0.0, 0, 0, 0
    while spent < seconds:
        i = (t + passes) % gen_steps
        q, kn, vn = q_all[i], kn_all[i], vn_all[i]
        for idx in order:
            l, b, h = units[idx]
            n = cache.length(l, b)
            s0 = cache.stream_slot(l, b, h)
            K = wl.to_numpy_storage(cache.k[s0:s0 + n])
            V = wl.to_numpy_storage(cache.v[s0:s0 + n])
            sc = cache.score[s0:s0 + n].cpu().numpy()
            ps = cache.pos[s0:s0 + n].cpu().numpy()
            qq = wl.to_numpy_storage(q[l, b, h * G:(h + 1) * G])
            kk = wl.to_numpy_storage(kn[l, b, h])
            vv = wl.to_numpy_storage(vn[l, b, h])
            t0 = time.perf_counter()
            u = orc.OracleUnit(K, V, sc, ps)
            u.append(kk, vv, w.context + t + passes)
            u.attend(qq)
            u.evict(int(budgets[l, b]))
            spent += time.perf_counter() - t0
            done += 1
            tokens += n + 1
            if spent >= seconds:
                break
        passes += 1
    if limiter is not None:
        limiter.restore_original_limits() if hasattr(limiter, "restore_original_limits") else None
    units_per_layer_step = w.batch * w.n_kv_heads
    # extrapolated by token count: the sample's tokens per second over the mean tokens of a layer-step
    mean_tokens_per_layer_step = float((budgets.astype("int64") + 1).sum()) * w.n_kv_heads / w.n_layers
    rate = (tokens / spent) / mean_tokens_per_layer_step
    return {"value": rate, "unit": "layer-steps/s", "cores": 1, "kind": "oracle",
            "sample": f"{done} (layer, sequence, KV-head) unit-steps ({len(units)} units per step, "
                      f"{passes} pass(es) with successive decode inputs), "
                      f"{spent:.1f} s of NumPy float64 on one thread, extrapolated by token count "
                      f"({units_per_layer_step} units per layer-step)"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
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
    W = max(args.warmup, 0)
    if args.evict_every > 1:
        W = max(W, args.evict_every)          # the warm-up ends with the first (prompt-sized) eviction
    K = args.steps if args.steps is not None else max(w.decode_steps - W, 1)
    L, B = w.n_layers, w.batch

    note(f"workload {w.name}: budgets")
    budgets, alloc = make_budgets(xkv, wl, w)
    every = max(args.evict_every, 1)
    if args.n_protect > 0:
        budgets = np.maximum(budgets, args.n_protect).astype(np.int32)
    caps = np.full((L, B), wl.round_up(w.context + every, 8), dtype=np.int32)
    cache = xkv.XkvCache(L, B, w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, caps)
    wl.fill_prompt_cache(w, cache.k, cache.v, cache.score, cache.pos, cache.region_off, cache.cap)
    cache.len[:] = w.context
    n_in = W + K + 1
    gen_steps = min(n_in, 256)
    q, kn, vn, pos_new = wl.decode_inputs(w, steps=gen_steps, device="cuda")
    out = torch.empty((L, B, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    ws = torch.empty(xkv.xkv_workspace_bytes(cache, L), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    pos_step = np.zeros(B, np.int32)

    alg_bytes = [0]

    state = {"cache": cache, "ws": ws}

    def step(t):
        i = t % gen_steps
        c = state["cache"]
        pos_step[:] = w.context + t
        alg_bytes[0] += algorithmic_bytes(w, c.len + 1)
        xkv.xkv_decode_attend_score(c, 0, L, q[i], kn[i], vn[i], pos_step, out, state["ws"], stream=stream)
        if (t + 1) % every == 0:
            xkv.xkv_evict_compact(c, 0, L, budgets, state["ws"], pool_size=args.pool_size,
                                  n_protect=args.n_protect, stream=stream)

    note("prompt cache filled; warm-up steps")
    t = 0
    step0_ms = None
    for _ in range(W):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        step(t)
        torch.cuda.synchronize()
        if t == 0:
            step0_ms = (time.perf_counter() - t0) * 1e3
        if t == every - 1:
            if not args.keep_prompt_arena:
                # the prompt-sized arena has done its job: continue in one sized by the budgets
                packed = repack(cache, budgets, slack=every)
                del ws, cache
                state["cache"] = None
                state["ws"] = None
                torch.cuda.empty_cache()
                cache = packed
                ws = torch.empty(xkv.xkv_workspace_bytes(cache, L), dtype=torch.uint8, device="cuda")
                state["cache"], state["ws"] = cache, ws
        t += 1


    torch.cuda.synchronize()
    note(f"timing {K} steps")
    alg_bytes[0] = 0
    t0 = time.perf_counter()
    for _ in range(K):
        step(t)
        t += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    alg_bytes_timed = alg_bytes[0]
    ms_per_step = elapsed / K * 1e3
    value = L * K / elapsed

    roofline = None
    steady = bool(np.all(cache.len.reshape(L, B) < budgets + every))
    if not args.no_roofline_pass:
        note("roofline pass")
        alg_bytes[0] = 0
        xkv.xkv_profile_enable(True)
        for _ in range(K):
            step(t)
            t += 1
        torch.cuda.synchronize()
        alg_bytes_step = alg_bytes[0] / K
        launches, total_ms = xkv.xkv_profile_read(0)
        sel_launches, sel_ms = xkv.xkv_profile_read(1)
        xkv.xkv_profile_enable(False)
        launches_per_step = launches / K
        bytes_per_launch = alg_bytes_step / launches_per_step
        achieved = bytes_per_launch / (total_ms / launches * 1e-3) / 1e9
        traffic = None
        tfile = os.path.join(ROOT, "profiles", f"decode_kernels_{w.name}_hbm_traffic.txt")
        if os.path.exists(tfile):
            for line in open(tfile):
                if line.startswith("traffic_bytes_per_launch:"):
                    traffic = float(line.split(":")[1])
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                    "kernel": ("attend_strip" if w.group <= 2 else "attend_gqa") +
                              " (K/V streaming kernel of xkv_decode_attend_score)",
                    "avg_launch_ms": total_ms / launches,
                    "launches_per_step": launches_per_step, "algorithmic_bytes_per_launch": bytes_per_launch,
                    "evict_select_avg_ms": (sel_ms / sel_launches) if sel_launches else None}

    # The same step captured once in a HIP graph and replayed (extra figure, not `value`: every
    # replay appends the captured step's token and position again).
    graph_ms = None
    if every == 1 and not args.no_graph:
        note("graph replay")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        gr = torch.cuda.CUDAGraph()
        i = t % gen_steps
        pos_step[:] = w.context + t
        with torch.cuda.stream(side):
            with torch.cuda.graph(gr, stream=side):
                xkv.xkv_decode_attend_score(cache, 0, L, q[i], kn[i], vn[i], pos_step, out, ws, stream=side)
                xkv.xkv_evict_compact(cache, 0, L, budgets, ws, pool_size=args.pool_size,
                                      n_protect=args.n_protect, stream=side)
        torch.cuda.current_stream().wait_stream(side)
        gr.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            gr.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / K * 1e3
        del gr

    # What a read-only kernel of the same shape reaches on this machine (context for the roofline fraction).
    ceiling = None
    if not args.no_roofline_pass:
        buf = cache.k
        per_wg = 128 * 1024
        nbytes = buf.numel() * buf.element_size() // per_wg * per_wg
        sink = torch.empty((nbytes // per_wg) * 1024, dtype=torch.float32, device="cuda")
        ceiling = {"bytes_per_launch": nbytes}
        # loads: non-temporal or ordinary; then non-temporal loads with 1.5 KB (a strip record) or 4 KB
        # (the logits of 256 slots at G = 4) stored per 128 KiB read, under the three store policies
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

    # Prefill-phase eviction (Alg. 2 as written, ows = 8, ps = 7), layer by layer as a
    # prefill would call it: one dense layer of the prompt at a time into a budget-sized cache.
    prefill = None
    if not args.no_prefill:
        note("prefill-phase eviction leg")
        ows, ps = 8, 7
        bud_p = np.maximum(budgets, ows)
        caps_p = ((np.minimum(bud_p, w.context).astype(np.int64) + 7) // 8 * 8).astype(np.int32)
        dst = xkv.XkvCache(L, B, w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, caps_p)
        ws_p = torch.empty(xkv.xkv_prefill_workspace_bytes(dst, 1, w.context, ows), dtype=torch.uint8, device="cuda")
        q_win, k_src, v_src = wl.dense_prompt_layer(w, 0, ows, device="cuda")
        xkv.xkv_prefill_evict(dst, 0, 1, q_win, k_src, v_src, w.context, ows, bud_p[0:1], ws_p, pool_size=ps,
                              stream=stream)                                 # warm-up
        torch.cuda.synchronize()
        xkv.xkv_profile_enable(True)
        t0 = time.perf_counter()
        for l in range(L):
            xkv.xkv_prefill_evict(dst, l, l + 1, q_win, k_src, v_src, w.context, ows, bud_p[l:l + 1], ws_p,
                                  pool_size=ps, stream=stream)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        n_stats, ms_stats = xkv.xkv_profile_read(2)
        xkv.xkv_profile_enable(False)
        row = w.head_dim * w.elem_bytes
        kept = np.minimum(bud_p, w.context).astype(np.int64)
        # K of the prompt read once, kept K and V rows read and written, score and pos written
        pre_bytes = int(L * B * w.n_kv_heads * w.context * row + kept.sum() * w.n_kv_heads * (4 * row + 8))
        k_pass_bytes = B * w.n_kv_heads * w.context * row
        prefill = {"ows": ows, "pool_size": ps, "ms_per_layer": dt / L * 1e3, "layers_per_s": L / dt,
                   "algorithmic_bytes_per_layer": pre_bytes / L, "hbm_gbs": pre_bytes / dt / 1e9,
                   "hbm_frac": pre_bytes / dt / 1e9 / HBM_PEAK_GBS,
                   "window_stats_avg_ms": ms_stats / n_stats if n_stats else None,
                   "window_stats_hbm_frac": (k_pass_bytes / (ms_stats / n_stats * 1e-3) / 1e9 / HBM_PEAK_GBS)
                   if n_stats else None,
                   "note": "the same dense layer is the source for every layer; budgets differ per layer"}
        del dst, ws_p, q_win, k_src, v_src

    cpu = None
    if args.cpu_seconds > 0:
        note("oracle on the host cores")
        cpu = cpu_baseline(w, wl, cache, budgets, (q, kn, vn, gen_steps), t, args.cpu_seconds)

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
                     "device_identical": bool(np.array_equal(dev_bud, budgets[:, 0])), "r_avg": alloc["r_avg"]}

    step_gbs = alg_bytes_timed / elapsed / 1e9
    line = {
        "metric": "decode attend+evict layer-steps/sec; achieved HBM GB/s vs MI355X peak",
        "value": value, "unit": "layer-steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "layers": L, "q_heads": w.n_q_heads, "kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "batch": B, "context": w.context,
                   "total_budget": int(budgets[:, 0].sum()), "budget_frac": w.budget_frac,
                   "budget_min": int(budgets.min()), "budget_max": int(budgets.max()),
                   "schedule": "every step, every layer: append, attend+score" +
                               (", evict to budget" if every == 1 else f"; every {every} steps: evict to budget"),
                   "pool_size": args.pool_size, "n_protect": args.n_protect, "attend_path": args.attend_path,
                   "arena": "prompt-sized" if args.keep_prompt_arena or W == 0 else "budget-sized after the first eviction",
                   "kv_arena_bytes": int(2 * cache.arena_slots * w.head_dim * w.elem_bytes),
                   "steady_state": steady},
        "step0_ms": step0_ms, "graph_replay_ms_per_step": graph_ms,
        "algorithmic_bytes_per_step": alg_bytes_timed / K,
        "step_hbm_gbs": step_gbs, "step_hbm_frac": step_gbs / HBM_PEAK_GBS,
        "roofline": roofline, "stream_read_ceiling": ceiling, "prefill_evict": prefill, "cpu_baseline": cpu,
        "allocator": allocator,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
