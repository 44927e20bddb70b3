"""GPU parity at the benchmark's full sizes, in the launch configuration
bench.py times: all layers in one call, prompt-sized arena for the first step,
budget-sized arena afterwards.  The oracle recomputes a seeded sample of
(layer, sequence, KV-head) units one by one; conservation of attention mass is
checked on every unit."""
import numpy as np
import pytest
import torch

import xkv_workloads as wl
from oracle import xkv_oracle as orc
from gpu_util import TOL, get_unit, rel_err, storage

pytestmark = pytest.mark.gpu


def unit_mass(cache):
    """Sum of the scores of every unit, [L, B, Hkv] (a plain device reduction)."""
    out = np.zeros((cache.n_layers, cache.batch, cache.n_kv_heads))
    for l in range(cache.n_layers):
        for b in range(cache.batch):
            n = cache.length(l, b)
            s0 = cache.stream_slot(l, b, 0)
            cap = int(cache.cap[l * cache.batch + b])
            blk = cache.score[s0:s0 + cap * cache.n_kv_heads].view(cache.n_kv_heads, cap)[:, :n]
            out[l, b] = blk.double().sum(dim=1).cpu().numpy()
    return out


def run_full(xkv, name, steps, n_sample, step_twin=False):
    """step_twin: from the second step on (budget-sized arena, steady state) a copy of the cache takes
    xkv_decode_step, the call bench.py times, and must equal the two calls' cache bit for bit."""
    w = wl.WORKLOADS[name]
    L, B, G = w.n_layers, w.batch, w.group
    if w.budget_rule == "dirichlet":
        budgets = np.ascontiguousarray(wl.dirichlet_budgets(L, B, w.context, w.total_budget, w.seed), dtype=np.int32)
        assert np.all(budgets.sum(axis=0) == w.total_budget)
        b1 = budgets[:, 0]
    else:
        curves = wl.zipf_importance_curves(L, w.context, w.seed)
        floor = [w.min_budget] * L if w.min_budget else None
        b1, ravg = xkv.xkv_allocate_budgets(curves, total_size=w.total_budget, min_budget=floor)
        assert int(b1.sum()) == w.total_budget
        budgets = np.repeat(b1.astype(np.int32)[:, None], B, axis=1)
    caps = np.full((L, B), (w.context + 1 + 7) // 8 * 8, dtype=np.int32)
    cache = xkv.XkvCache(L, B, w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, caps)
    print(f"{name}: filling {2 * cache.arena_slots * w.head_dim * w.elem_bytes / 1e9:.1f} GB of K/V", flush=True)
    wl.fill_prompt_cache(w, cache.k, cache.v, cache.score, cache.pos, cache.region_off, cache.cap)
    cache.len[:] = w.context
    ws = torch.empty(xkv.xkv_workspace_bytes(cache, L), dtype=torch.uint8, device="cuda")
    q, kn, vn, pos_new = wl.decode_inputs(w, steps=steps, device="cuda")
    out = torch.empty((L, B, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")

    r = np.random.default_rng(w.seed)
    lmax, lmin = int(np.argmax(b1)), int(np.argmin(b1))
    units = [(lmax, 0, 0), (lmin, 0, w.n_kv_heads - 1)]
    while len(units) < n_sample:
        u = (int(r.integers(L)), int(r.integers(B)), int(r.integers(w.n_kv_heads)))
        if u not in units:
            units.append(u)
    orcs = {u: orc.OracleUnit(*get_unit(cache, *u)) for u in units}
    evicted = np.zeros((L, B, w.n_kv_heads))
    twin, out_b, one_kernel_steps = None, None, 0
    for step in range(steps):
        print(f"{name}: step {step}", flush=True)
        if twin is not None:
            xkv.xkv_profile_enable(True)
            xkv.xkv_decode_step(twin, 0, L, q[step], kn[step], vn[step], pos_new[step], out_b, budgets, ws_b)
            torch.cuda.synchronize()
            one_kernel_steps += 1 if xkv.xkv_profile_read(3)[0] > 0 else 0
            xkv.xkv_profile_enable(False)
        xkv.xkv_decode_attend_score(cache, 0, L, q[step], kn[step], vn[step], pos_new[step], out, ws)
        torch.cuda.synchronize()
        o_host = out.cpu().numpy()
        for (l, b, h), u in orcs.items():
            u.append(storage(kn[step, l, b, h]), storage(vn[step, l, b, h]), pos_new[step, b])
            o, _ = u.attend(storage(q[step, l, b, h * G:(h + 1) * G]))
            K, V, sc, pos = get_unit(cache, l, b, h)
            for g in range(G):
                e = rel_err(o_host[l, b, h * G + g], o[g])
                assert e <= TOL[w.dtype], f"step {step} unit {(l, b, h)} out err {e}"
            e = rel_err(sc, u.score)
            assert e <= TOL[w.dtype], f"step {step} unit {(l, b, h)} score err {e}"
            assert np.array_equal(pos, u.pos)
            u.score = sc
        before = unit_mass(cache)
        kept = torch.zeros(cache.arena_slots, dtype=torch.int32, device="cuda")
        xkv.xkv_evict_compact(cache, 0, L, budgets, ws, kept_idx_out=kept)
        torch.cuda.synchronize()
        after = unit_mass(cache)
        evicted += before - after
        # every query head spends exactly one unit of probability per step
        total = after + evicted
        assert np.max(np.abs(total - G * (step + 1))) <= 2e-3 * G * (step + 1), "attention mass is conserved"
        assert np.array_equal(cache.len.reshape(L, B), np.minimum(budgets, w.context + step + 1))
        for (l, b, h), u in orcs.items():
            ki = u.evict(int(budgets[l, b]))
            s0 = cache.stream_slot(l, b, h)
            assert np.array_equal(kept[s0:s0 + u.n].cpu().numpy(), ki), f"step {step} unit {(l, b, h)} kept_idx"
            K, V, sc, pos = get_unit(cache, l, b, h)
            assert np.array_equal(K, u.K) and np.array_equal(V, u.V)
            assert np.array_equal(sc, u.score) and np.array_equal(pos, u.pos)
        del kept
        if twin is not None:
            assert np.array_equal(twin.len, cache.len)
            assert torch.equal(twin.k, cache.k) and torch.equal(twin.v, cache.v), f"step {step}: twin K/V"
            assert torch.equal(twin.score, cache.score) and torch.equal(twin.pos, cache.pos), f"step {step}: twin"
            assert rel_err(out_b.cpu().numpy(), o_host) <= 1e-5
        if step == 0:
            small = cache.resized(((budgets.astype(np.int64) + 1 + 7) // 8 * 8).astype(np.int32))
            del cache, ws
            torch.cuda.empty_cache()
            cache = small
            ws = torch.empty(xkv.xkv_workspace_bytes(cache, L), dtype=torch.uint8, device="cuda")
            if step_twin:
                torch.cuda.synchronize()
                twin = xkv.XkvCache(L, B, w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, cache.cap.reshape(L, B), zero=False)
                twin.k.copy_(cache.k); twin.v.copy_(cache.v); twin.score.copy_(cache.score); twin.pos.copy_(cache.pos)
                twin.len[:] = cache.len
                ws_b = torch.empty(xkv.xkv_workspace_bytes(twin, L), dtype=torch.uint8, device="cuda")
                out_b = torch.empty_like(out)
    return one_kernel_steps


@pytest.fixture(params=[2, 1], ids=["fused", "two-kernels"])
def attend_path(request, xkv):
    xkv.xkv_configure(xkv.XKV_CFG_ATTEND_PATH, request.param)
    yield request.param
    xkv.xkv_configure(xkv.XKV_CFG_ATTEND_PATH, 0)


def test_llama2_7b_4k_full_size(xkv, attend_path):
    run_full(xkv, "llama2_7b_4k", steps=3, n_sample=8)


def test_llama2_7b_32k_full_size(xkv, attend_path):
    run_full(xkv, "llama2_7b_32k", steps=3, n_sample=8)


@pytest.mark.parametrize("name", ["llama2_7b_4k", "llama2_7b_32k"])
def test_decode_step_at_full_size(xkv, name):
    """The call the benchmark times, xkv_decode_step, on the budget-sized arena: three steady-state steps
    on a copy of the cache, each through the kernel that updates the scores and evicts, bit for bit equal
    to the two calls (which are held against the oracle as above)."""
    assert run_full(xkv, name, steps=4, n_sample=4, step_twin=True) == 3


def test_mistral_7b_gqa_b32_full_size(xkv):
    """Batched GQA (G = 4) through the matrix-core kernel: 8 launches per call, per-sequence budgets."""
    run_full(xkv, "mistral_7b_gqa_b32", steps=2, n_sample=6)


def test_llama3_70b_128k_full_size(xkv):
    """G = 8, 128k-token streams, 172 GB of K/V in the prompt-sized arena."""
    run_full(xkv, "llama3_70b_128k", steps=2, n_sample=5)
