"""GPU parity over multi-step decode runs, in lockstep with the oracle.

A one-ulp difference in a score can flip an eviction and fork the two caches,
so every step (1) compares out and score within tolerance, (2) feeds the GPU's
score array to the oracle's selection and requires identical kept indices,
(3) continues the oracle from the GPU's post-eviction state."""
import numpy as np
import pytest
import torch

import xkv_workloads as wl
from oracle import xkv_oracle as orc
from gpu_util import TOL, get_unit, rel_err, storage

pytestmark = pytest.mark.gpu


def build(xkv, w, budgets, cap_extra=8):
    caps = np.full((w.n_layers, w.batch), w.context + cap_extra, dtype=np.int32)
    cache = xkv.XkvCache(w.n_layers, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, caps)
    wl.fill_prompt_cache(w, cache.k, cache.v, cache.score, cache.pos, cache.region_off, cache.cap)
    cache.len[:] = w.context
    ws = torch.empty(xkv.xkv_workspace_bytes(cache, w.n_layers), dtype=torch.uint8, device="cuda")
    return cache, ws


def lockstep(xkv, w, budgets, units, steps, pool=1, protect=0, first_evict_step=0):
    cache, ws = build(xkv, w, budgets)
    G = w.group
    q, kn, vn, pos_new = wl.decode_inputs(w, steps=steps, device="cuda")
    out = torch.empty((w.n_layers, w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    kept = torch.zeros(cache.arena_slots, dtype=torch.int32, device="cuda")
    orcs = {u: orc.OracleUnit(*get_unit(cache, *u)) for u in units}
    evicted_mass = {u: 0.0 for u in units}
    own_scores = {}
    for step in range(steps):
        xkv.xkv_decode_attend_score(cache, 0, w.n_layers, q[step], kn[step], vn[step], pos_new[step], out, ws)
        torch.cuda.synchronize()
        o_host = out.cpu().numpy()
        for (l, b, h), u in orcs.items():
            u.append(storage(kn[step, l, b, h]), storage(vn[step, l, b, h]), pos_new[step, b])
            o, _ = u.attend(storage(q[step, l, b, h * G:(h + 1) * G]))
            K, V, sc, pos = get_unit(cache, l, b, h)
            assert sc.shape[0] == u.n
            for g in range(G):
                e = rel_err(o_host[l, b, h * G + g], o[g])
                assert e <= TOL[w.dtype], f"step {step} unit {(l, b, h)} out err {e}"
            e = rel_err(sc, u.score)
            assert e <= TOL[w.dtype], f"step {step} unit {(l, b, h)} score err {e}"
            assert np.array_equal(pos, u.pos) and np.array_equal(K, u.K) and np.array_equal(V, u.V)
            total = float(sc.astype(np.float64).sum()) + evicted_mass[(l, b, h)]
            assert abs(total - G * (step + 1)) <= 1e-4 * G * (step + 1), "attention mass is conserved"
            own_scores[(l, b, h)] = u.score.copy()
            u.score = sc                       # select from the same score array
        if step < first_evict_step:
            continue
        xkv.xkv_evict_compact(cache, 0, w.n_layers, budgets, ws, pool_size=pool, n_protect=protect,
                              kept_idx_out=kept)
        torch.cuda.synchronize()
        for (l, b, h), u in orcs.items():
            before = float(u.score.astype(np.float64).sum())
            n_before, pos_before = u.n, u.pos.copy()
            ki = u.evict(int(budgets[l, b]), pool, protect)
            check_valid_top_set(own_scores[(l, b, h)], pos_before, ki, pool, protect, TOL[w.dtype])
            evicted_mass[(l, b, h)] += before - float(u.score.astype(np.float64).sum())
            s0 = cache.stream_slot(l, b, h)
            assert cache.length(l, b) == u.n
            assert np.array_equal(kept[s0:s0 + u.n].cpu().numpy(), ki), f"step {step} unit {(l, b, h)} kept_idx"
            K, V, sc, pos = get_unit(cache, l, b, h)
            assert np.array_equal(K, u.K) and np.array_equal(V, u.V)
            assert np.array_equal(sc, u.score) and np.array_equal(pos, u.pos)
            assert sorted(pos.tolist()) == sorted(u.pos.tolist())
    return cache


def check_valid_top_set(own_score, pos, kept_idx, pool, protect, tol):
    """The kept slots against the scores the oracle computed itself for this step (nothing of
    the device in them): up to the tolerance they are a top set of the unprotected slots."""
    n = own_score.shape[0]
    kept = np.zeros(n, bool)
    kept[kept_idx] = True
    if kept.all():
        return
    key = orc.pooled_keys(own_score, pool).astype(np.float64)
    free = np.ones(n, bool)
    if protect > 0:
        free = pos < 1 + int(pos.max()) - protect
        assert kept[~free].all()
    if not (kept & free).any():
        return
    slack = tol * pool * float(key.max())
    assert key[kept & free].min() >= key[~kept].max() - 2 * slack


def all_units(w):
    return [(l, b, h) for l in range(w.n_layers) for b in range(w.batch) for h in range(w.n_kv_heads)]


@pytest.fixture(params=[2, 1], ids=["fused", "two-kernels"])
def attend_path(request, xkv):
    xkv.xkv_configure(xkv.XKV_CFG_ATTEND_PATH, request.param)
    yield request.param
    xkv.xkv_configure(xkv.XKV_CFG_ATTEND_PATH, 0)


def test_tiny_fp32_full_run_every_unit(xkv, attend_path):
    """The small fp32 configuration: 4 layers, 4 heads, d 64, prompt 512, 16
    steps, budgets 384/256/128/64 (sum 832), sinks at tokens 0-3."""
    w = wl.WORKLOADS["tiny_f32"]
    budgets = np.asarray(w.fixed_budgets, np.int32).reshape(w.n_layers, 1)
    assert budgets.sum() == 832
    cache = lockstep(xkv, w, budgets, all_units(w), w.decode_steps)
    assert cache.len.tolist() == [384, 256, 128, 64]
    # the sink tokens (key norm x4) draw attention mass and survive
    for h in range(4):
        _, _, _, pos = get_unit(cache, 0, 0, h)
        assert len(set(pos.tolist()) & {0, 1, 2, 3}) >= 1


def test_tiny_paper_defaults_window_and_pooling(xkv, attend_path):
    """Observation window 8 and pooling width 7 (the paper's default setting):
    the first eviction waits for 8 decode steps, the newest 8 tokens are kept."""
    w = wl.WORKLOADS["tiny_f32"]
    budgets = np.asarray(w.fixed_budgets, np.int32).reshape(w.n_layers, 1)
    lockstep(xkv, w, budgets, all_units(w), 12, pool=7, protect=8, first_evict_step=7)


def test_gqa_bf16_batched_sampled_units(xkv, attend_path):
    """Mistral-shaped geometry at reduced size: GQA 32/8, batch 3, per-sequence budgets."""
    w = wl.scaled(wl.WORKLOADS["mistral_7b_gqa_b32"], n_layers=3, batch=3, context=1500, decode_steps=4)
    budgets = wl.dirichlet_budgets(w.n_layers, w.batch, w.context, int(0.3 * w.n_layers * w.context), w.seed)
    r = np.random.default_rng(0)
    units = [all_units(w)[i] for i in r.choice(len(all_units(w)), size=12, replace=False)]
    lockstep(xkv, w, budgets, units, w.decode_steps)
