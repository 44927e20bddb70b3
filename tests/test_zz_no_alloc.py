"""GPU test of xkv_decode_attend_score_noalloc, the entry point that allocates
nothing: called through the C ABI (ctypes on the raw symbol), compared with
xkv_decode_attend_score on the same inputs.  Both run the same kernels, so
outputs, scores and the appended rows must agree bit for bit; the first call is
also held against the oracle at the stated tolerance.  Two calls in a row, the
second on a smaller input, because every call on a GPU shares one scratch array
that keeps the previous call's contents."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import xkv_oracle as orc
from gpu_util import TOL, get_unit, random_fill, rel_err, storage

pytestmark = pytest.mark.gpu


def _call_both(xkv, dtype, d, Hq, Hkv, L, B, lens, seed, check_oracle):
    lib = xkv.load()
    lens = np.asarray(lens, np.int32).reshape(L, B)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    g = torch.Generator(device="cpu").manual_seed(seed + 1)
    q = torch.randn((L, B, Hq, d), generator=g).to(tdt).cuda()
    kn = torch.randn((L, B, Hkv, d), generator=g).to(tdt).cuda()
    vn = torch.randn((L, B, Hkv, d), generator=g).to(tdt).cuda()
    pos_new = (np.arange(B, dtype=np.int32) + 777)
    results = []
    for which in ("workspace", "noalloc"):
        cache = xkv.XkvCache(L, B, Hq, Hkv, d, dtype, lens + 3)
        random_fill(cache, lens, seed)
        before = {(l, b, h): get_unit(cache, l, b, h) for l in range(L) for b in range(B) for h in range(Hkv)}
        out = torch.full((L, B, Hq, d), float("nan"), dtype=torch.float32, device="cuda")
        stream = torch.cuda.current_stream().cuda_stream or None
        print(f"case {which} dtype={dtype} d={d} Hq={Hq} Hkv={Hkv} lens={lens.tolist()}", flush=True)
        if which == "workspace":
            ws = torch.empty(xkv.xkv_workspace_bytes(cache, L), dtype=torch.uint8, device="cuda")
            st = lib.xkv_decode_attend_score(C.byref(cache.struct), 0, L, q.data_ptr(), kn.data_ptr(), vn.data_ptr(),
                                             pos_new.ctypes.data, 0.0, out.data_ptr(), ws.data_ptr(), ws.numel(),
                                             stream)
        else:
            st = lib.xkv_decode_attend_score_noalloc(C.byref(cache.struct), 0, L, q.data_ptr(), kn.data_ptr(),
                                                     vn.data_ptr(), pos_new.ctypes.data, 0.0, out.data_ptr(), stream)
        assert st == 0, xkv.status_string(st)
        torch.cuda.synchronize()
        assert np.array_equal(cache.len.reshape(L, B), lens + 1)
        results.append((out.cpu().numpy(), cache.k.cpu().view(torch.uint8).numpy(), cache.v.cpu().view(torch.uint8).numpy(),
                        cache.score.cpu().numpy(), cache.pos.cpu().numpy()))
        if which == "noalloc" and check_oracle:
            G = Hq // Hkv
            o_host = results[-1][0]
            for (l, b, h), (K, V, score, pos) in before.items():
                u = orc.OracleUnit(K, V, score, pos)
                u.append(storage(kn[l, b, h]), storage(vn[l, b, h]), pos_new[b])
                o, _ = u.attend(storage(q[l, b, h * G:(h + 1) * G]))
                _, _, s2, _ = get_unit(cache, l, b, h)
                for gq in range(G):
                    assert rel_err(o_host[l, b, h * G + gq], o[gq]) <= TOL[dtype]
                assert rel_err(s2, u.score) <= TOL[dtype]
    for a, b in zip(*results):
        assert np.array_equal(a, b, equal_nan=True)


@pytest.mark.parametrize("dtype,d,Hq,Hkv", [("bf16", 128, 4, 4), ("bf16", 128, 8, 2), ("f32", 64, 4, 2)])
def test_noalloc_matches_workspace_entry_point_twice(xkv, dtype, d, Hq, Hkv):
    # first call: several strips per stream and ragged tails; second call: smaller, over the same scratch array
    _call_both(xkv, dtype, d, Hq, Hkv, 3, 2, [[5000, 0], [257, 9000], [1, 4096]], seed=11, check_oracle=True)
    _call_both(xkv, dtype, d, Hq, Hkv, 2, 1, [[300], [17]], seed=12, check_oracle=True)


def test_noalloc_refuses_what_does_not_fit(xkv):
    """More strip records than the fixed array holds: XKV_ERR_CAPACITY, nothing enqueued, lengths untouched."""
    lib = xkv.load()
    L, B, Hq, Hkv, d = 1, 1, 32, 32, 128
    n = 800000                                  # 32 heads x 800 k slots x 2 bytes of logit records > 32 MiB
    cache = xkv.XkvCache(L, B, Hq, Hkv, d, "bf16", [[n + 8]])
    cache.len[:] = n
    q = torch.zeros((L, B, Hq, d), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((L, B, Hq, d), dtype=torch.float32, device="cuda")
    st = lib.xkv_decode_attend_score_noalloc(C.byref(cache.struct), 0, L, q.data_ptr(), None, None, None, 0.0,
                                             out.data_ptr(), None)
    assert st == -3, xkv.status_string(st)
    assert int(cache.len[0]) == n
