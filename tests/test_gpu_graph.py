"""A steady-state decode step (append + attention/scoring + eviction) captured in a HIP graph:
the library launches on the capturing stream, copies nothing from the host and records no memset
nodes, so replays must reproduce the eager result bit for bit, also with eager work in between."""
import numpy as np
import pytest
import torch

from gpu_util import random_fill

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("one_call", [False, True], ids=["two-calls", "decode-step"])
@pytest.mark.parametrize("dtype,d,Hq,Hkv,many", [("bf16", 128, 4, 4, False), ("bf16", 128, 8, 2, False),
                                                 ("f32", 64, 4, 4, False), ("bf16", 128, 8, 2, True),
                                                 ("bf16", 128, 2, 2, True)])
def test_captured_step_replays_like_eager(xkv, dtype, d, Hq, Hkv, many, one_call):
    """many: more regions than the kernel arguments hold, so the graph also holds the launches
    that write the geometry tables.  one_call: the step is xkv_decode_step (eager and captured)."""
    def run_step(c, q_, kn_, vn_, out_, ws_, stream=None):
        if one_call:
            xkv.xkv_decode_step(c, 0, L, q_, kn_, vn_, pos_new, out_, budgets, ws_, stream=stream)
        else:
            xkv.xkv_decode_attend_score(c, 0, L, q_, kn_, vn_, pos_new, out_, ws_, stream=stream)
            xkv.xkv_evict_compact(c, 0, L, budgets, ws_, stream=stream)

    if many:
        L, B = 3, 50
        budgets = np.random.default_rng(4).integers(8, 200, size=(L, B)).astype(np.int32)
    else:
        L, B = 3, 2
        budgets = np.array([[700, 300], [64, 1500], [256, 257]], np.int32)
    caps = budgets + 8

    def fresh():
        cache = xkv.XkvCache(L, B, Hq, Hkv, d, dtype, caps)
        random_fill(cache, budgets, seed=5)
        return cache

    g = torch.Generator(device="cpu").manual_seed(9)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    steps = 4
    qs = torch.randn((steps, L, B, Hq, d), generator=g).to(tdt).cuda()
    kns = torch.randn((steps, L, B, Hkv, d), generator=g).to(tdt).cuda()
    vns = torch.randn((steps, L, B, Hkv, d), generator=g).to(tdt).cuda()
    pos_new = (9000 + np.arange(B)).astype(np.int32)

    # eager reference: the state after every step
    ref = fresh()
    ws_ref = torch.empty(xkv.xkv_workspace_bytes(ref, L), dtype=torch.uint8, device="cuda")
    out_ref = torch.empty((L, B, Hq, d), dtype=torch.float32, device="cuda")
    states = []
    for s in range(steps):
        run_step(ref, qs[s], kns[s], vns[s], out_ref, ws_ref)
        torch.cuda.synchronize()
        states.append((out_ref.clone(), ref.k.clone(), ref.score.clone(), ref.pos.clone()))

    # captured: static input buffers, one graph, replayed once per step
    cache = fresh()
    ws = torch.empty(xkv.xkv_workspace_bytes(cache, L), dtype=torch.uint8, device="cuda")
    out = torch.empty((L, B, Hq, d), dtype=torch.float32, device="cuda")
    q, kn, vn = qs[0].clone(), kns[0].clone(), vns[0].clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    snapshot = (cache.k.clone(), cache.v.clone(), cache.score.clone(), cache.pos.clone())
    with torch.cuda.stream(side):
        # warm-up launch outside the capture (loads the code objects), then restore the state
        run_step(cache, q, kn, vn, out, ws, stream=side)
        side.synchronize()
        for dst, src in zip((cache.k, cache.v, cache.score, cache.pos), snapshot):
            dst.copy_(src)
        side.synchronize()
        assert np.array_equal(cache.len.reshape(L, B), budgets)       # the step returns to its lengths
        with torch.cuda.graph(graph, stream=side):
            run_step(cache, q, kn, vn, out, ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    assert np.array_equal(cache.len.reshape(L, B), budgets)
    for s in range(steps):
        q.copy_(qs[s]); kn.copy_(kns[s]); vn.copy_(vns[s])
        graph.replay()
        torch.cuda.synchronize()
        # eager work between replays
        junk = (torch.randn(1 << 16, device="cuda") * 2).sum().item()
        assert np.isfinite(junk)
        o, k, sc, ps = states[s]
        assert torch.equal(out, o), f"replay {s}: output"
        assert torch.equal(cache.k, k) and torch.equal(cache.score, sc) and torch.equal(cache.pos, ps), f"replay {s}: cache"
