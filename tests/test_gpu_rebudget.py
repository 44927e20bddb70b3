"""GPU parity for re-budgeting during decode: xkv_cache_importance against the
oracle (bit for bit: fp32 adds in head order), and the whole flow
decode -> importance -> xkv_allocate_budgets_device -> xkv_repack ->
xkv_evict_compact to the new budgets -> decode, checked against the oracle step
by step in lockstep."""
import numpy as np
import pytest
import torch

import xkv_workloads as wl
from oracle import xkv_oracle as orc
from gpu_util import TOL, get_unit, random_fill, rel_err, storage

pytestmark = pytest.mark.gpu


def oracle_vectors(cache, n_pos):
    """The oracle's vector of every (layer, sequence) from the device cache's pos and score arrays."""
    out = np.zeros((cache.n_layers, cache.batch, n_pos), np.float32)
    for l in range(cache.n_layers):
        for b in range(cache.batch):
            units = [get_unit(cache, l, b, h) for h in range(cache.n_kv_heads)]
            out[l, b] = orc.cache_importance([u[3] for u in units], [u[2] for u in units], n_pos)
    return out


@pytest.mark.parametrize("dtype,d,Hkv,L,B,nmax,n_pos", [
    ("f32", 64, 3, 2, 2, 700, 710),          # one range of positions
    ("bf16", 128, 2, 2, 1, 20000, 20003),    # several ranges
    ("bf16", 128, 4, 3, 2, 500, 300),        # tokens beyond n_pos are left out
    ("bf16", 64, 1, 40, 30, 60, 70),         # more regions (1200) than one launch describes
])
def test_cache_importance_matches_the_oracle(xkv, dtype, d, Hkv, L, B, nmax, n_pos):
    r = np.random.default_rng(nmax)
    lens = r.integers(0, nmax + 1, size=(L, B)).astype(np.int32)
    lens.reshape(-1)[0] = nmax
    if lens.size > 1:
        lens.reshape(-1)[1] = 0
    cache = xkv.XkvCache(L, B, Hkv, Hkv, d, dtype, lens + 2)
    random_fill(cache, lens, 31)             # distinct positions in [0, n + 3) per stream, scores in [0, 1)
    w_dev = torch.full((L, B, n_pos), float("nan"), dtype=torch.float32, device="cuda")
    print(f"case importance dtype={dtype} Hkv={Hkv} L={L} B={B} nmax={nmax} n_pos={n_pos}", flush=True)
    xkv.xkv_cache_importance(cache, 0, L, n_pos, w_dev)
    torch.cuda.synchronize()
    assert np.array_equal(w_dev.cpu().numpy().view(np.uint32), oracle_vectors(cache, n_pos).view(np.uint32))


def test_layer_range_and_errors(xkv):
    lens = np.array([[50], [70], [30]], np.int32)
    cache = xkv.XkvCache(3, 1, 2, 2, 64, "f32", lens + 2)
    random_fill(cache, lens, 5)
    w_dev = torch.zeros((1, 1, 80), dtype=torch.float32, device="cuda")
    xkv.xkv_cache_importance(cache, 1, 2, 80, w_dev)
    torch.cuda.synchronize()
    assert np.array_equal(w_dev.cpu().numpy()[0, 0], oracle_vectors(cache, 80)[1, 0])
    with pytest.raises(xkv.XkvError) as e:
        xkv.xkv_cache_importance(cache, 0, 3, 0, w_dev)
    assert e.value.status == -1
    with pytest.raises(xkv.XkvError) as e:
        xkv.xkv_cache_importance(cache, 0, 3, 80, None)
    assert e.value.status == -1


@pytest.mark.parametrize("dtype,d,Hq,Hkv", [("f32", 64, 4, 2), ("bf16", 128, 8, 2)])
def test_rebudget_flow_in_lockstep_with_the_oracle(xkv, dtype, d, Hq, Hkv):
    L, B, T, G = 4, 2, 400, Hq // Hkv
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], n_layers=L, batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d,
                  dtype=dtype, context=T, decode_steps=10, fixed_budgets=None)
    budgets = np.array([[300, 280], [200, 220], [120, 100], [60, 80]], np.int32)
    total = budgets.sum(axis=0)                                   # per sequence: kept when re-budgeting
    cache = xkv.XkvCache(L, B, Hq, Hkv, d, dtype, np.full((L, B), T + 8, np.int32))
    wl.fill_prompt_cache(w, cache.k, cache.v, cache.score, cache.pos, cache.region_off, cache.cap)
    cache.len[:] = T
    q, kn, vn, pos_new = wl.decode_inputs(w, steps=10, device="cuda")
    out = torch.empty((L, B, Hq, d), dtype=torch.float32, device="cuda")
    units = [(l, b, h) for l in range(L) for b in range(B) for h in range(Hkv)]
    orcs = {u: orc.OracleUnit(*get_unit(cache, *u)) for u in units}
    state = {"cache": cache, "ws": torch.empty(xkv.xkv_workspace_bytes(cache, L), dtype=torch.uint8, device="cuda")}

    def evict(bud, tag):
        c = state["cache"]
        kept = torch.zeros(c.arena_slots, dtype=torch.int32, device="cuda")
        xkv.xkv_evict_compact(c, 0, L, bud, state["ws"], kept_idx_out=kept)
        torch.cuda.synchronize()
        for (l, b, h), u in orcs.items():
            ki = u.evict(int(bud[l, b]))
            s0 = c.stream_slot(l, b, h)
            assert c.length(l, b) == u.n, tag
            assert np.array_equal(kept[s0:s0 + u.n].cpu().numpy(), ki), f"{tag} unit {(l, b, h)} kept_idx"
            K, V, sc, pos = get_unit(c, l, b, h)
            assert np.array_equal(K, u.K) and np.array_equal(V, u.V) and np.array_equal(sc, u.score)
            assert np.array_equal(pos, u.pos)

    def decode_step(step, bud):
        c = state["cache"]
        xkv.xkv_decode_attend_score(c, 0, L, q[step], kn[step], vn[step], pos_new[step], out, state["ws"])
        torch.cuda.synchronize()
        o_host = out.cpu().numpy()
        for (l, b, h), u in orcs.items():
            u.append(storage(kn[step, l, b, h]), storage(vn[step, l, b, h]), pos_new[step, b])
            o, _ = u.attend(storage(q[step, l, b, h * G:(h + 1) * G]))
            K, V, sc, pos = get_unit(c, l, b, h)
            for g in range(G):
                assert rel_err(o_host[l, b, h * G + g], o[g]) <= TOL[dtype], f"step {step} out"
            assert rel_err(sc, u.score) <= TOL[dtype], f"step {step} score"
            assert np.array_equal(pos, u.pos) and np.array_equal(K, u.K)
            u.score = sc                      # lockstep: decisions are taken on the device's scores
        evict(bud, f"step {step}")

    for step in range(5):
        decode_step(step, budgets)

    # ---- re-budget: importance -> allocation (device) -> move -> evict ----------------
    c = state["cache"]
    n_pos = T + 5
    w_dev = torch.empty((L, B, n_pos), dtype=torch.float32, device="cuda")
    xkv.xkv_cache_importance(c, 0, L, n_pos, w_dev)
    torch.cuda.synchronize()
    w_host = w_dev.cpu().numpy()
    w_ref = np.zeros_like(w_host)
    for l in range(L):
        for b in range(B):
            w_ref[l, b] = orc.cache_importance([orcs[l, b, h].pos for h in range(Hkv)],
                                               [orcs[l, b, h].score for h in range(Hkv)], n_pos)
    assert np.array_equal(w_host.view(np.uint32), w_ref.view(np.uint32))
    aws = torch.empty(xkv.xkv_allocate_device_workspace_bytes(L, n_pos), dtype=torch.uint8, device="cuda")
    floor = [16] * L
    new_budgets = np.zeros((L, B), np.int32)
    for b in range(B):
        got, ravg = xkv.xkv_allocate_budgets_device(w_dev[:, b], L, n_pos, B * n_pos, int(total[b]), aws,
                                                    min_budget=floor)
        ref, ravg_ref = orc.allocate_budgets([w_ref[l, b] for l in range(L)], total_size=int(total[b]),
                                             min_budget=floor)
        assert np.array_equal(got, np.asarray(ref)), (b, got, ref)
        assert abs(ravg - ravg_ref) < 1e-9
        new_budgets[:, b] = got
    assert np.array_equal(new_budgets.sum(axis=0), total)
    assert not np.array_equal(new_budgets, budgets)               # the allocation really moved
    # layers that are to grow need room: a cache with the new capacities
    new_caps = (np.maximum(new_budgets, c.len.reshape(L, B)) + 8).astype(np.int32)
    moved = c.resized(new_caps)
    torch.cuda.synchronize()
    for (l, b, h), u in orcs.items():
        K, V, sc, pos = get_unit(moved, l, b, h)
        assert np.array_equal(K, u.K) and np.array_equal(V, u.V) and np.array_equal(sc, u.score)
        assert np.array_equal(pos, u.pos)
    state["cache"] = moved
    state["ws"] = torch.empty(xkv.xkv_workspace_bytes(moved, L), dtype=torch.uint8, device="cuda")
    evict(new_budgets, "re-budget")                               # shrinking layers shrink at once
    assert np.array_equal(moved.len.reshape(L, B), np.minimum(new_budgets, budgets))

    # ---- decoding goes on under the new budgets; growing layers fill up ----------------
    for step in range(5, 10):
        decode_step(step, new_budgets)
    assert np.all(moved.len.reshape(L, B) <= new_budgets)
    grown = new_budgets > budgets
    assert np.array_equal(moved.len.reshape(L, B)[grown], np.minimum(new_budgets, budgets + 5)[grown])
