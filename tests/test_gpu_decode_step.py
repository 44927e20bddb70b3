"""GPU parity: xkv_decode_step against the two calls it stands for (cache state bit for bit) and,
over several steps, against the oracle in lockstep."""
import numpy as np
import pytest
import torch

from oracle import xkv_oracle as orc
from gpu_util import TOL, get_unit, random_fill, rel_err, storage

pytestmark = pytest.mark.gpu


def twin_caches(xkv, L, B, Hq, Hkv, d, dtype, caps, lens, seed, ties):
    a = xkv.XkvCache(L, B, Hq, Hkv, d, dtype, caps)
    b = xkv.XkvCache(L, B, Hq, Hkv, d, dtype, caps)
    random_fill(a, lens, seed, ties=ties)
    b.k.copy_(a.k); b.v.copy_(a.v); b.score.copy_(a.score); b.pos.copy_(a.pos)
    b.len[:] = a.len
    return a, b


def run_both(xkv, dtype, d, G, lens, evict, append, seed, pool=1, protect=0, ties=False, expect_one_kernel=None,
             Hkv=2):
    """evict[l][b]: tokens to evict from the length after the append (budget = that length - evict)."""
    lens = np.asarray(lens, np.int32)
    L, B = lens.shape
    after = lens + (1 if append else 0)
    budgets = np.maximum(after - np.asarray(evict, np.int32), protect).astype(np.int32)
    caps = after + 2
    a, b = twin_caches(xkv, L, B, Hkv * G, Hkv, d, dtype, caps, lens, seed, ties)
    g = torch.Generator(device="cpu").manual_seed(seed + 1)
    tdt = a.torch_dtype
    q = torch.randn((L, B, Hkv * G, d), generator=g).to(tdt).cuda()
    kn = torch.randn((L, B, Hkv, d), generator=g).to(tdt).cuda() if append else None
    vn = torch.randn((L, B, Hkv, d), generator=g).to(tdt).cuda() if append else None
    pos_new = np.arange(1000, 1000 + B, dtype=np.int32) if append else None
    out_a = torch.zeros((L, B, Hkv * G, d), dtype=torch.float32, device="cuda")
    out_b = torch.zeros_like(out_a)
    ws = torch.empty(xkv.xkv_workspace_bytes(a, L), dtype=torch.uint8, device="cuda")
    kept_a = torch.full((a.k.shape[0],), -7, dtype=torch.int32, device="cuda")
    kept_b = torch.full_like(kept_a, -7)
    xkv.xkv_decode_attend_score(a, 0, L, q, kn, vn, pos_new, out_a, ws)
    xkv.xkv_evict_compact(a, 0, L, budgets, ws, pool_size=pool, n_protect=protect, kept_idx_out=kept_a)
    xkv.xkv_profile_enable(True)
    xkv.xkv_decode_step(b, 0, L, q, kn, vn, pos_new, out_b, budgets, ws, pool_size=pool, n_protect=protect,
                        kept_idx_out=kept_b)
    torch.cuda.synchronize()
    launches, _ = xkv.xkv_profile_read(3)
    xkv.xkv_profile_enable(False)
    if expect_one_kernel is not None:
        assert (launches > 0) == expect_one_kernel, f"score-and-evict kernel launches: {launches}"
    assert np.array_equal(a.len, b.len)
    assert torch.equal(a.k, b.k) and torch.equal(a.v, b.v) and torch.equal(a.pos, b.pos)
    assert torch.equal(a.score, b.score)
    for l in range(L):
        for bb in range(B):
            kk = a.length(l, bb)
            for h in range(Hkv):
                s0 = a.stream_slot(l, bb, h)
                assert torch.equal(kept_a[s0:s0 + kk], kept_b[s0:s0 + kk])
    oa, ob = out_a.cpu().numpy(), out_b.cpu().numpy()
    assert np.all(np.isfinite(ob))
    assert rel_err(ob, oa) <= 1e-5


@pytest.mark.parametrize("dtype,d,G", [("bf16", 128, 1), ("f32", 64, 1), ("bf16", 128, 2), ("f32", 128, 2),
                                       ("bf16", 64, 1), ("f32", 64, 4), ("bf16", 64, 8), ("bf16", 128, 4),
                                       ("bf16", 128, 8)])
@pytest.mark.parametrize("append", [True, False])
def test_step_equals_the_two_calls_in_the_steady_state(xkv, dtype, d, G, append):
    """Streams of 0, 1, a few, ragged and several strips of slots; 0 to 8 evictions each."""
    print(f"case step dtype={dtype} d={d} G={G} append={append}", flush=True)
    lens = [[0, 1, 9], [255, 256, 257], [700, 5000, 1030]]
    evict = [[0, 1 if append else 0, 8], [1, 0, 3], [8, 2, 1]]
    one = not (dtype == "bf16" and d == 128 and G >= 4)     # the matrix-core path keeps its own kernels
    run_both(xkv, dtype, d, G, lens, evict, append, seed=200 + G, expect_one_kernel=one)
    # equal scores everywhere: the evicted ones are the highest slots among the smallest
    run_both(xkv, dtype, d, G, lens, evict, append, seed=210 + G, ties=True, expect_one_kernel=one)


def test_step_keeps_nothing_or_everything(xkv):
    """Budget 0 (the stream is emptied) and budgets beyond the length."""
    lens = [[40, 300]]
    run_both(xkv, "bf16", 128, 1, lens, [[41, 0]], True, seed=230, expect_one_kernel=True)
    run_both(xkv, "f32", 64, 2, lens, [[-5, -100]], True, seed=231, expect_one_kernel=True)


def test_step_falls_back_to_the_two_calls(xkv):
    """More than 8 evictions in some stream: the two calls' kernels, same result, no score-and-evict launch."""
    run_both(xkv, "bf16", 128, 1, [[300, 900]], [[9, 1]], True, seed=240, expect_one_kernel=False)
    run_both(xkv, "f32", 64, 2, [[300, 900]], [[2, 500]], False, seed=241, pool=3, protect=2, expect_one_kernel=False)


@pytest.mark.parametrize("dtype,d,G", [("bf16", 128, 1), ("f32", 64, 2), ("f32", 128, 4)])
@pytest.mark.parametrize("pool,protect", [(7, 8), (3, 0), (1, 5), (63, 1)])
def test_step_with_pooling_and_protected_tokens(xkv, dtype, d, G, pool, protect):
    """The paper's settings (pooling 7, the 8 most recent positions never evicted) and others: keys derived
    from the scores the step has just written."""
    print(f"case step derived keys dtype={dtype} d={d} G={G} pool={pool} protect={protect}", flush=True)
    lens = [[8, 9, 40], [255, 256, 257], [700, 5000, 1030]]
    evict = [[1, 1, 0], [1, 0, 1], [1, 1, 1]]
    run_both(xkv, dtype, d, G, lens, evict, True, seed=280 + G, pool=pool, protect=protect, expect_one_kernel=True)
    run_both(xkv, dtype, d, G, lens, evict, False, seed=290 + G, pool=pool, protect=protect, ties=True,
             expect_one_kernel=True)
    # more than one eviction with derived keys: the two calls' kernels
    run_both(xkv, dtype, d, G, lens, [[1, 1, 8], [1, 0, 3], [8, 2, 1]], True, seed=295 + G, pool=pool, protect=protect,
             expect_one_kernel=False)


def test_long_streams_and_both_workgroup_sizes(xkv):
    """Two long streams per layer (few streams: the 1024-thread workgroups) and the same lengths in a
    call of 512 streams (256-thread workgroups)."""
    run_both(xkv, "bf16", 128, 1, [[20001, 12000]], [[1, 8]], True, seed=250, expect_one_kernel=True)
    run_both(xkv, "f32", 64, 2, [[16385]], [[2]], False, seed=251, expect_one_kernel=True)
    lens = np.full((8, 16), 40, np.int32)
    lens[3, 5] = 9000
    lens[7, 15] = 4097
    evict = np.ones((8, 16), np.int32)
    evict[3, 5] = 7
    run_both(xkv, "bf16", 128, 1, lens, evict, True, seed=252, expect_one_kernel=True, Hkv=4)


@pytest.mark.parametrize("dtype,d,G", [("bf16", 128, 1), ("f32", 64, 2), ("bf16", 128, 4)])
def test_calls_on_more_regions_than_the_kernel_arguments_hold(xkv, dtype, d, G):
    """256 (layer, sequence) regions: the geometry tables and the keep counts travel through device memory."""
    r = np.random.default_rng(270 + G)
    lens = r.integers(0, 60, size=(16, 16)).astype(np.int32)
    lens[2, 3] = 5000
    lens[9, 0] = 0
    evict = r.integers(0, 9, size=(16, 16)).astype(np.int32)
    evict = np.minimum(evict, lens + 1)
    one = G < 4
    run_both(xkv, dtype, d, G, lens, evict, True, seed=271 + G, expect_one_kernel=one)
    run_both(xkv, dtype, d, G, lens, np.minimum(evict, lens), False, seed=272 + G, ties=True, expect_one_kernel=one)


@pytest.mark.parametrize("dtype,d,G", [("bf16", 128, 1), ("f32", 64, 2), ("bf16", 128, 8)])
def test_steps_in_lockstep_with_the_oracle(xkv, dtype, d, G):
    """Twelve decode steps (append, attention, scoring, eviction back to a fixed budget) on twin
    caches.  The first takes the two calls and is held against the oracle unit by unit: outputs and
    scores within the tolerance, then the oracle's selection on the device's own scores, whose
    result (kept tokens, their order, scores) must be the device's bit for bit.  The second takes
    xkv_decode_step and must equal the first bit for bit after every step."""
    L, B, Hkv = 2, 2, 2
    lens = np.array([[300, 40], [1030, 257]], np.int32)
    budgets = lens.copy()                                  # steady state: one in, one out
    a, b = twin_caches(xkv, L, B, Hkv * G, Hkv, d, dtype, lens + 2, lens, 260, False)
    units = {(l, s, h): orc.OracleUnit(*get_unit(a, l, s, h)) for l in range(L) for s in range(B) for h in range(Hkv)}
    ws = torch.empty(xkv.xkv_workspace_bytes(a, L), dtype=torch.uint8, device="cuda")
    out_a = torch.zeros((L, B, Hkv * G, d), dtype=torch.float32, device="cuda")
    out_b = torch.zeros_like(out_a)
    g = torch.Generator(device="cpu").manual_seed(261)
    tdt = a.torch_dtype
    xkv.xkv_profile_enable(True)
    for step in range(12):
        q = torch.randn((L, B, Hkv * G, d), generator=g).to(tdt).cuda()
        kn = torch.randn((L, B, Hkv, d), generator=g).to(tdt).cuda()
        vn = torch.randn((L, B, Hkv, d), generator=g).to(tdt).cuda()
        pos_new = np.array([5000 + step, 6000 + step], np.int32)
        xkv.xkv_decode_attend_score(a, 0, L, q, kn, vn, pos_new, out_a, ws)
        torch.cuda.synchronize()
        o_host = out_a.cpu().numpy()
        for (l, s, h), u in units.items():
            u.append(storage(kn[l, s, h]), storage(vn[l, s, h]), int(pos_new[s]))
            o, _ = u.attend(storage(q[l, s, h * G:(h + 1) * G]))
            assert rel_err(o_host[l, s, h * G:(h + 1) * G], o) <= TOL[dtype]
            _, _, sc, _ = get_unit(a, l, s, h)
            assert rel_err(sc, u.score) <= TOL[dtype]
            u.score = sc                                   # the selection is taken on the device's scores
        xkv.xkv_evict_compact(a, 0, L, budgets, ws)
        xkv.xkv_decode_step(b, 0, L, q, kn, vn, pos_new, out_b, budgets, ws)
        torch.cuda.synchronize()
        for (l, s, h), u in units.items():
            u.evict(int(budgets[l, s]))
            K, V, sc, pos = get_unit(a, l, s, h)
            assert np.array_equal(K, u.K) and np.array_equal(V, u.V)
            assert np.array_equal(sc, u.score) and np.array_equal(pos, u.pos)
        assert np.array_equal(a.len, b.len)
        assert torch.equal(a.k, b.k) and torch.equal(a.v, b.v) and torch.equal(a.pos, b.pos)
        assert torch.equal(a.score, b.score), f"step {step}"
        assert rel_err(out_b.cpu().numpy(), o_host) <= 1e-5
    launches, _ = xkv.xkv_profile_read(3)
    xkv.xkv_profile_enable(False)
    assert launches == (12 if G < 4 else 0)
