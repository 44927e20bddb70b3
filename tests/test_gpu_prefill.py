"""GPU parity: xkv_prefill_evict against the oracle's Alg. 2, unit by unit.

The attention mass w is compared within the floating-point tolerance; the
selection is an integer decision taken on w, so the oracle repeats it on the
device's own fp32 w and everything after it (kept positions, gathered rows,
scores) must then match bit for bit."""
import numpy as np
import pytest
import torch

from oracle import xkv_oracle as orc
from gpu_util import TOL, get_unit, rel_err, storage

pytestmark = pytest.mark.gpu


def check_selection_is_valid_for(w_ref, kept_pos, t, ows, ps, tol):
    """Independent of anything the device computed: against the oracle's own masses the kept
    candidates must be a top set up to the tolerance (several sets are correct when keys lie
    that close to the threshold)."""
    tc = t - ows
    kc = len(kept_pos) - ows
    if kc <= 0 or kc >= tc:
        return
    key = orc.pooled_keys(w_ref[:tc].astype(np.float32), ps).astype(np.float64)
    kept = np.zeros(tc, bool)
    kept[kept_pos[:kc]] = True
    slack = tol * ps * float(key.max())
    assert key[kept].min() >= key[~kept].max() - 2 * slack


def window_lse_of(q_win, k_src, G, tb, scale, units=None):
    """The oracle's row normalisers of every stream as the fp32 tensor the lse entry points take
    ([layers, B, Hq, ows]); streams outside `units` get NaN (the test does not look at them)."""
    nl, B, Hq, ows, _ = q_win.shape
    Hkv = Hq // G
    out = np.full((nl, B, Hq, ows), np.nan, np.float32)
    for l in range(nl):
        for b in range(B):
            for h in range(Hkv):
                if units is not None and (l, b, h) not in units:
                    continue
                K = storage(k_src[l, b, h])[:int(tb[b])]
                q = storage(q_win[l, b, h * G:(h + 1) * G])
                out[l, b, h * G:(h + 1) * G] = orc.window_row_lse(q, K, None if scale == 0.0 else scale)
    return out


def run_prefill(xkv, dtype, d, Hq, Hkv, L, B, t, ows, ps, budgets, seed, scale=0.0, layer_range=None,
                heavy=True, with_w=True, check_units=None, t_per_seq=None, given_lse=False):
    """t_per_seq: prompt length of every sequence (rows beyond it hold NaN: they must never be read).
    given_lse: the call takes the window rows' normalisers from the oracle (xkv_prefill_evict_lse)."""
    budgets = np.asarray(budgets, np.int32).reshape(L, B)
    tb = np.full(B, t, np.int64) if t_per_seq is None else np.asarray(t_per_seq, np.int64)
    caps = np.minimum(budgets, tb[None, :]) + 3
    cache = xkv.XkvCache(L, B, Hq, Hkv, d, dtype, caps)
    G = Hq // Hkv
    l0, l1 = layer_range or (0, L)
    nl = l1 - l0
    g = torch.Generator(device="cpu").manual_seed(seed)
    tdt = cache.torch_dtype
    k_src = torch.randn((nl, B, Hkv, t, d), generator=g)
    if heavy:                                   # a few dominant tokens, as in the paper's heat map
        hot = torch.randperm(t, generator=g)[:max(1, t // 50)]
        k_src[:, :, :, hot, :] *= 3.0
    v_src = torch.randn((nl, B, Hkv, t, d), generator=g)
    for b in range(B):
        k_src[:, b, :, int(tb[b]):, :] = float("nan")
        v_src[:, b, :, int(tb[b]):, :] = float("nan")
    k_src = k_src.to(tdt).cuda()
    v_src = v_src.to(tdt).cuda()
    q_win = torch.randn((nl, B, Hq, ows, d), generator=g).to(tdt).cuda()
    ws = torch.empty(xkv.xkv_prefill_workspace_bytes(cache, L, t, ows), dtype=torch.uint8, device="cuda")
    w_out = torch.full((nl, B, Hkv, t), float("nan"), dtype=torch.float32, device="cuda") if with_w else None
    cache.len[:] = 1                            # whatever was there is overwritten
    if given_lse:
        assert layer_range is None
        lse = torch.from_numpy(window_lse_of(q_win, k_src, G, tb, scale)).cuda()
        xkv.xkv_prefill_evict_lse(cache, l0, l1, q_win, k_src, v_src, t, ows, budgets[l0:l1], lse, ws,
                                  pool_size=ps, softmax_scale=scale, w_out=w_out, t_per_seq=t_per_seq)
    else:
        xkv.xkv_prefill_evict(cache, l0, l1, q_win, k_src, v_src, t, ows, budgets[l0:l1], ws, pool_size=ps,
                              softmax_scale=scale, w_out=w_out, t_per_seq=t_per_seq)
    torch.cuda.synchronize()
    assert not xkv.xkv_fused_status()           # no wait of a one-launch selection gave up
    w_dev = w_out.cpu().numpy() if with_w else None
    worst = 0.0
    for l in range(L):
        for b in range(B):
            if not (l0 <= l < l1):
                assert cache.length(l, b) == 1
                continue
            ts = int(tb[b])                      # this sequence's prompt
            kk = min(int(budgets[l, b]), ts)
            assert cache.length(l, b) == kk
            for h in range(Hkv):
                if check_units is not None and (l, b, h) not in check_units:
                    continue
                K = storage(k_src[l - l0, b, h])[:ts]
                V = storage(v_src[l - l0, b, h])[:ts]
                q = storage(q_win[l - l0, b, h * G:(h + 1) * G])
                w_ref = orc.window_attention_mass(q, K, None if scale == 0.0 else scale)
                K2, V2, s2, p2 = get_unit(cache, l, b, h)
                if with_w:
                    wd = w_dev[l - l0, b, h][:ts]
                    assert np.all(np.isfinite(wd))
                    assert np.all(np.isnan(w_dev[l - l0, b, h][ts:]))      # nothing written past the prompt
                    worst = max(worst, rel_err(wd, w_ref))
                    assert abs(float(wd.astype(np.float64).sum()) - G * ows) < 1e-3 * G * ows
                    Ko, Vo, so, po, _ = orc.prefill_evict(q, K, V, kk, ows, ps, w=wd)
                    assert np.array_equal(p2, po), f"kept positions differ in unit {(l, b, h)}"
                    assert np.array_equal(K2, Ko) and np.array_equal(V2, Vo) and np.array_equal(s2, so)
                    check_selection_is_valid_for(w_ref, p2, ts, ows, ps, TOL[dtype])
                else:
                    # without w_out: what is unique is checked (the window, order, rows, scores
                    # within tolerance) and the kept set is valid for scores within tolerance
                    assert np.all(np.diff(p2) > 0) and np.array_equal(p2[kk - ows:], np.arange(ts - ows, ts))
                    assert np.array_equal(K2, K[p2]) and np.array_equal(V2, V[p2])
                    worst = max(worst, rel_err(s2, w_ref[p2]))
    assert worst <= TOL[dtype], f"w rel err {worst}"
    return worst


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128), ("bf16", 64), ("f32", 128)])
@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_shapes_groups_and_ragged_prompts(xkv, dtype, d, G):
    """Prompt lengths that end inside a 16-row group; budgets from window-only to everything."""
    Hkv = 2
    for t, ows, ps in [(300, 8, 7), (257, 5, 1), (64, 8, 3)]:
        if ows * G > 64:
            ows = 64 // G
        budgets = [[ows, t + 5], [t // 3, t - 1]]
        print(f"case dtype={dtype} d={d} G={G} t={t} ows={ows} ps={ps}", flush=True)
        run_prefill(xkv, dtype, d, Hkv * G, Hkv, 2, 2, t, ows, ps, budgets, seed=100 + G + t)


def test_window_covers_whole_prompt_and_single_row_window(xkv):
    run_prefill(xkv, "f32", 64, 2, 2, 1, 1, 8, 8, 1, [[8]], seed=1)        # no candidate at all
    run_prefill(xkv, "bf16", 128, 4, 2, 1, 2, 500, 1, 7, [[100, 1]], seed=2)   # ows = 1: a decode query


def test_ties_go_to_the_lower_position(xkv):
    """Identical keys for all tokens: uniform attention, so candidates tie in
    bulk and the kept ones must be the first."""
    L, B, Hkv, t, ows, d = 1, 1, 1, 700, 4, 64
    cache = xkv.XkvCache(L, B, 1, Hkv, d, "f32", [[300]])
    k_src = torch.ones((1, 1, 1, t, d), device="cuda")
    v_src = torch.randn((1, 1, 1, t, d), device="cuda")
    q_win = torch.randn((1, 1, 1, ows, d), device="cuda")
    ws = torch.empty(xkv.xkv_prefill_workspace_bytes(cache, 1, t, ows), dtype=torch.uint8, device="cuda")
    xkv.xkv_prefill_evict(cache, 0, 1, q_win, k_src, v_src, t, ows, np.array([[200]], np.int32), ws)
    torch.cuda.synchronize()
    _, _, s2, p2 = get_unit(cache, 0, 0, 0)
    assert p2.tolist() == list(range(196)) + list(range(696, 700))
    expect = sum(1.0 / (t - ows + r + 1) for r in range(ows))
    assert abs(float(s2[0]) - expect) < 1e-6


def test_layer_subrange_scale_and_no_w_out(xkv):
    run_prefill(xkv, "bf16", 128, 8, 2, 3, 2, 1000, 8, 7, [[100, 200], [300, 50], [999, 1000]], seed=5,
                scale=0.11, layer_range=(1, 3))
    run_prefill(xkv, "f32", 64, 4, 4, 2, 1, 400, 8, 7, [[100], [37]], seed=6, with_w=False)


def test_long_prompt_many_strips_and_launch_groups(xkv):
    """A 20k-token prompt (several strips per stream) and more regions than one launch describes."""
    o = run_prefill(xkv, "bf16", 128, 8, 2, 1, 2, 20011, 8, 7, [[4000, 6001]], seed=7)
    print("long prompt w rel err", o, flush=True)
    r = np.random.default_rng(0)
    budgets = r.integers(8, 300, size=(3, 50))
    run_prefill(xkv, "bf16", 128, 2, 1, 3, 50, 333, 8, 7, budgets, seed=8)


def test_decode_continues_on_a_prefilled_cache(xkv):
    """The decode step runs on what the prefill call left: scores keep accumulating."""
    L, B, Hq, Hkv, d, t, ows = 2, 1, 4, 2, 128, 600, 8
    budgets = np.array([[150], [90]], np.int32)
    cache = xkv.XkvCache(L, B, Hq, Hkv, d, "bf16", budgets + 2)
    g = torch.Generator(device="cpu").manual_seed(3)
    k_src = torch.randn((L, B, Hkv, t, d), generator=g).bfloat16().cuda()
    v_src = torch.randn((L, B, Hkv, t, d), generator=g).bfloat16().cuda()
    q_win = torch.randn((L, B, Hq, ows, d), generator=g).bfloat16().cuda()
    ws = torch.empty(max(xkv.xkv_prefill_workspace_bytes(cache, L, t, ows), xkv.xkv_workspace_bytes(cache, L)),
                     dtype=torch.uint8, device="cuda")
    xkv.xkv_prefill_evict(cache, 0, L, q_win, k_src, v_src, t, ows, budgets, ws, pool_size=7)
    torch.cuda.synchronize()
    units = {(l, h): orc.OracleUnit(*get_unit(cache, l, 0, h)) for l in range(L) for h in range(Hkv)}
    q = torch.randn((L, B, Hq, d), generator=g).bfloat16().cuda()
    kn = torch.randn((L, B, Hkv, d), generator=g).bfloat16().cuda()
    vn = torch.randn((L, B, Hkv, d), generator=g).bfloat16().cuda()
    out = torch.empty((L, B, Hq, d), dtype=torch.float32, device="cuda")
    xkv.xkv_decode_attend_score(cache, 0, L, q, kn, vn, np.array([t], np.int32), out, ws)
    xkv.xkv_evict_compact(cache, 0, L, budgets, ws, n_protect=ows)
    torch.cuda.synchronize()
    for (l, h), u in units.items():
        u.append(storage(kn[l, 0, h]), storage(vn[l, 0, h]), t)
        o, _ = u.attend(storage(q[l, 0, h * 2:(h + 1) * 2]))
        K2, V2, s2, p2 = get_unit(cache, l, 0, h)
        assert rel_err(out[l, 0, h * 2:(h + 1) * 2].cpu().numpy(), o) <= TOL["bf16"]
        assert len(p2) == budgets[l, 0] and t in p2.tolist()


def test_full_size_layer_of_the_long_context_workload(xkv):
    """One layer of the 32k workload as the benchmark's prefill leg calls it (32 heads, t = 32768,
    register-resident keys in the selection); four sampled heads against the oracle."""
    units = {(0, 0, h) for h in (0, 7, 18, 31)}
    e = run_prefill(xkv, "bf16", 128, 32, 32, 1, 1, 32768, 8, 7, [[6554]], seed=31, check_units=units)
    print("32k layer w rel err", e, flush=True)


def test_full_size_layer_of_the_128k_gqa_workload(xkv):
    """One layer of the 128k GQA workload (G = 8: 64 window rows per KV head, t = 131072, keys through
    the workspace), two sequences with the largest and the smallest budget; three sampled units."""
    units = {(0, 0, 0), (0, 1, 7), (0, 0, 5)}
    e = run_prefill(xkv, "bf16", 128, 64, 8, 1, 2, 131072, 8, 7, [[19661, 256]], seed=32, check_units=units)
    print("128k layer w rel err", e, flush=True)


def test_full_size_layers_with_given_normalisers(xkv):
    """The same two full-size layers through xkv_prefill_evict_lse (one K pass)."""
    e = run_prefill(xkv, "bf16", 128, 32, 32, 1, 1, 32768, 8, 7, [[6554]], seed=31,
                    check_units={(0, 0, h) for h in (3, 30)}, given_lse=True)
    print("32k layer, given normalisers, w rel err", e, flush=True)
    e = run_prefill(xkv, "bf16", 128, 64, 8, 1, 1, 131072, 8, 7, [[19661]], seed=33,
                    check_units={(0, 0, 2), (0, 0, 7)}, given_lse=True)
    print("128k layer, given normalisers, w rel err", e, flush=True)


@pytest.mark.parametrize("ps", [1, 5])
def test_long_stream_selection_split_over_workgroups_with_bulk_ties(xkv, ps):
    """Few long streams take the selection that is split over several workgroups.  Equal keys
    everywhere make every candidate tie, across the workgroups' chunks too: the kept ones must be
    the first.  (With pooling the two ends of the candidate vector have smaller keys.)"""
    t, ows, d, budget = 40005, 4, 64, 20004
    cache = xkv.XkvCache(1, 1, 1, 1, d, "f32", [[budget + 4]])
    k_src = torch.ones((1, 1, 1, t, d), device="cuda")
    v_src = torch.randn((1, 1, 1, t, d), device="cuda")
    q_win = torch.randn((1, 1, 1, ows, d), device="cuda")
    ws = torch.empty(xkv.xkv_prefill_workspace_bytes(cache, 1, t, ows), dtype=torch.uint8, device="cuda")
    w_out = torch.empty((1, 1, 1, t), dtype=torch.float32, device="cuda")
    xkv.xkv_prefill_evict(cache, 0, 1, q_win, k_src, v_src, t, ows, np.array([[budget]], np.int32), ws,
                          pool_size=ps, w_out=w_out)
    torch.cuda.synchronize()
    K2, V2, s2, p2 = get_unit(cache, 0, 0, 0)
    wd = w_out.cpu().numpy()[0, 0, 0]
    ref = orc.prefill_select(wd, ows, budget, ps)
    assert np.array_equal(p2, ref)
    half = ps // 2
    assert p2[0] == half and p2[budget - ows - 1] == half + budget - ows - 1     # a prefix, after the weak edge
    assert np.array_equal(V2, storage(v_src[0, 0, 0])[p2])


def test_long_streams_split_selection_random_scores(xkv):
    o = run_prefill(xkv, "bf16", 128, 4, 2, 1, 2, 50003, 8, 7, [[12345, 49000]], seed=41)
    print("split selection w rel err", o, flush=True)
    run_prefill(xkv, "f32", 64, 2, 2, 1, 1, 33000, 8, 1, [[8]], seed=42)        # window only


@pytest.mark.parametrize("dtype,d,G,ows", [("bf16", 128, 1, 8), ("bf16", 128, 4, 8), ("f32", 64, 2, 5),
                                          ("bf16", 64, 8, 8), ("f32", 128, 1, 16)])
def test_given_row_normalisers_read_k_once(xkv, dtype, d, G, ows):
    """xkv_prefill_evict_lse: the masses from the caller's normalisers (here the oracle's) must be
    the softmax masses, ragged prompts and a non-default scale included."""
    print(f"case lse dtype={dtype} d={d} G={G} ows={ows}", flush=True)
    run_prefill(xkv, dtype, d, 2 * G, 2, 2, 3, 1203, ows, 7, [[300, 1203, 40], [ows, 700, 999]], seed=120 + G,
                given_lse=True, t_per_seq=[1203, 900, ows + 1])
    run_prefill(xkv, dtype, d, 2 * G, 2, 1, 1, 700, ows, 1, [[100]], seed=130 + G, scale=0.21, given_lse=True,
                with_w=False)


def test_given_row_normalisers_are_used_as_they_are(xkv):
    """Normalisers raised by ln 2 halve every mass (the library does not normalise again), and
    the importance vectors of the mini-prefill take them the same way."""
    L, B, Hq, Hkv, d, t, ows, ps = 1, 2, 4, 2, 128, 900, 8, 5
    G = Hq // Hkv
    cache = xkv.XkvCache(L, B, Hq, Hkv, d, "bf16", [[8, 8]])
    g = torch.Generator(device="cpu").manual_seed(140)
    k_src = torch.randn((L, B, Hkv, t, d), generator=g).bfloat16().cuda()
    q_win = torch.randn((L, B, Hq, ows, d), generator=g).bfloat16().cuda()
    lse = window_lse_of(q_win, k_src, G, [t, t], 0.0)
    ws = torch.empty(xkv.xkv_prefill_workspace_bytes(cache, L, t, ows), dtype=torch.uint8, device="cuda")
    w_a = torch.empty((L, B, t - ows), dtype=torch.float32, device="cuda")
    w_b = torch.empty_like(w_a)
    w_c = torch.empty_like(w_a)
    xkv.xkv_window_importance(cache, 0, L, q_win, k_src, t, ows, w_a, ws, pool_size=ps)
    xkv.xkv_window_importance_lse(cache, 0, L, q_win, k_src, t, ows, torch.from_numpy(lse).cuda(), w_b, ws,
                                  pool_size=ps)
    xkv.xkv_window_importance_lse(cache, 0, L, q_win, k_src, t, ows,
                                  torch.from_numpy(lse + np.float32(np.log(2.0))).cuda(), w_c, ws, pool_size=ps)
    torch.cuda.synchronize()
    a, b, c = (x.cpu().numpy() for x in (w_a, w_b, w_c))
    for s in range(B):
        q = storage(q_win[0, s]).reshape(Hkv, G, ows, d)
        ref = orc.window_importance(q, storage(k_src[0, s]), ps)
        assert rel_err(a[0, s], ref) <= TOL["bf16"] and rel_err(b[0, s], ref) <= TOL["bf16"]
        assert rel_err(c[0, s], 0.5 * ref) <= TOL["bf16"]


def test_one_launch_selection_give_up_is_reported(xkv):
    """Failure handling of the one-launch selection, forced from the host: with a poll limit of
    zero every workgroup gives up its first wait unpolled.  The kernels must still end normally,
    the status call must report it, the regions of the streams concerned keep what they held,
    and a stream that needs no selection (budget >= prompt) is filled all the same.  With the
    default limit the same call then completes and matches the oracle."""
    t, ows, ps, d = 20000, 8, 7, 64
    budgets = np.array([[5000, 20000]], np.int32)
    cache = xkv.XkvCache(1, 2, 1, 1, d, "f32", budgets + 2)
    g = torch.Generator(device="cpu").manual_seed(97)
    k_src = torch.randn((1, 2, 1, t, d), generator=g).cuda()
    v_src = torch.randn((1, 2, 1, t, d), generator=g).cuda()
    q_win = torch.randn((1, 2, 1, ows, d), generator=g).cuda()
    ws = torch.empty(xkv.xkv_prefill_workspace_bytes(cache, 1, t, ows), dtype=torch.uint8, device="cuda")
    cache.k.fill_(7.0)
    cache.pos.fill_(-5)
    xkv.xkv_configure(xkv.XKV_CFG_FUSED_SPIN_LIMIT, 0)
    try:
        print("case one-launch selection give-up, poll limit 0", flush=True)
        xkv.xkv_prefill_evict(cache, 0, 1, q_win, k_src, v_src, t, ows, budgets, ws, pool_size=ps)
        gave_up = xkv.xkv_fused_status()
    finally:
        xkv.xkv_configure(xkv.XKV_CFG_FUSED_SPIN_LIMIT, -1)
    assert gave_up
    assert cache.length(0, 0) == 5000 and cache.length(0, 1) == 20000
    K0, _, _, p0 = get_unit(cache, 0, 0, 0)
    assert np.all(K0 == 7.0) and np.all(p0 == -5)                     # untouched
    K1, V1, _, p1 = get_unit(cache, 0, 1, 0)
    assert np.array_equal(p1, np.arange(t)) and np.array_equal(K1, storage(k_src[0, 1, 0]))
    assert np.array_equal(V1, storage(v_src[0, 1, 0]))
    w_out = torch.empty((1, 2, 1, t), dtype=torch.float32, device="cuda")
    xkv.xkv_prefill_evict(cache, 0, 1, q_win, k_src, v_src, t, ows, budgets, ws, pool_size=ps, w_out=w_out)
    assert not xkv.xkv_fused_status()
    wd = w_out.cpu().numpy()[0, 0, 0]
    K0, V0, s0, p0 = get_unit(cache, 0, 0, 0)
    ref = orc.prefill_select(wd, ows, 5000, ps)
    assert np.array_equal(p0, ref)
    assert np.array_equal(K0, storage(k_src[0, 0, 0])[ref]) and np.array_equal(V0, storage(v_src[0, 0, 0])[ref])
    assert np.array_equal(s0, wd[ref])


@pytest.mark.parametrize("dtype,d,G", [("bf16", 128, 4), ("f32", 64, 1), ("bf16", 128, 1)])
def test_batch_of_prompts_of_different_lengths(xkv, dtype, d, G):
    """Every sequence has its own prompt length; the rows past it hold NaN and must not be read.
    Lengths end inside a 16-row group, equal the window, fill all rows."""
    t, ows = 1500, 8
    tps = [1500, 8, 777, 1001]
    budgets = [[300, 8, 800, 50], [1500, 100, 9, 1001]]
    run_prefill(xkv, dtype, d, 2 * G, 2, 2, 4, t, ows, 7, budgets, seed=70 + G, t_per_seq=tps)


def test_different_lengths_in_the_split_selection_and_score_vectors(xkv):
    """Long prompts of different lengths (selection split over workgroups), and the allocator's
    per-sequence score vectors for them."""
    t, ows, ps, Hq, Hkv, d = 40000, 8, 7, 4, 2, 128
    tps = [40000, 33333]
    run_prefill(xkv, "bf16", d, Hq, Hkv, 1, 2, t, ows, ps, [[9000, 33000]], seed=81, t_per_seq=tps)
    cache = xkv.XkvCache(1, 2, Hq, Hkv, d, "bf16", [[8, 8]])
    g = torch.Generator(device="cpu").manual_seed(82)
    k_src = torch.randn((1, 2, Hkv, t, d), generator=g)
    k_src[0, 1, :, tps[1]:, :] = float("nan")
    k_src = k_src.bfloat16().cuda()
    q_win = torch.randn((1, 2, Hq, ows, d), generator=g).bfloat16().cuda()
    ws = torch.empty(xkv.xkv_prefill_workspace_bytes(cache, 1, t, ows), dtype=torch.uint8, device="cuda")
    w_layer = torch.full((1, 2, t - ows), float("nan"), dtype=torch.float32, device="cuda")
    xkv.xkv_window_importance(cache, 0, 1, q_win, k_src, t, ows, w_layer, ws, pool_size=ps, t_per_seq=tps)
    torch.cuda.synchronize()
    got = w_layer.cpu().numpy()
    for b in range(2):
        tc = tps[b] - ows
        q = storage(q_win[0, b]).reshape(Hkv, Hq // Hkv, ows, d)
        ref = orc.window_importance(q, storage(k_src[0, b])[:, :tps[b]], ps)
        assert rel_err(got[0, b, :tc], ref) <= TOL["bf16"]
        assert np.all(np.isnan(got[0, b, tc:]))
