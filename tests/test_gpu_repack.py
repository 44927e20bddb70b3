"""GPU test of xkv_repack: bit-exact against slicing the arenas."""
import numpy as np
import pytest
import torch

from gpu_util import random_fill

pytestmark = pytest.mark.gpu


def _check_copy(src, dst, zeroed=True):
    assert np.array_equal(dst.len, src.len)
    sk, sv = src.k.view(torch.int16).cpu().numpy(), src.v.view(torch.int16).cpu().numpy()
    dk, dv = dst.k.view(torch.int16).cpu().numpy(), dst.v.view(torch.int16).cpu().numpy()
    ss, sp = src.score.cpu().numpy(), src.pos.cpu().numpy()
    ds, dp = dst.score.cpu().numpy(), dst.pos.cpu().numpy()
    touched = np.zeros(max(dst.arena_slots, 1), bool)
    for l in range(src.n_layers):
        for b in range(src.batch):
            n = src.length(l, b)
            for h in range(src.n_kv_heads):
                a, d = src.stream_slot(l, b, h), dst.stream_slot(l, b, h)
                assert np.array_equal(dk[d:d + n], sk[a:a + n]) and np.array_equal(dv[d:d + n], sv[a:a + n])
                assert np.array_equal(ds[d:d + n].view(np.uint32), ss[a:a + n].view(np.uint32))
                assert np.array_equal(dp[d:d + n], sp[a:a + n])
                touched[d:d + n] = True
    if not zeroed:
        return
    # nothing beyond the live slots was written: the new arenas start as zeros
    assert not dk[~touched].any() and not dv[~touched].any() and not ds[~touched].any() and not dp[~touched].any()


@pytest.mark.parametrize("dtype,d,Hkv,L,B", [("bf16", 128, 2, 3, 2), ("f32", 64, 3, 2, 2), ("bf16", 64, 1, 40, 30)])
def test_repack_matches_slicing(xkv, dtype, d, Hkv, L, B):
    """Ragged lengths with empty streams, a partial block, exactly one block and several; the last case has
    more regions (1200) than one launch describes."""
    r = np.random.default_rng(L * 100 + B)
    lens = r.integers(0, 90, size=(L, B)).astype(np.int32)
    lens.reshape(-1)[:4] = [0, 255, 256, 1500]
    src = xkv.XkvCache(L, B, Hkv * 2, Hkv, d, dtype, lens + r.integers(0, 9, size=(L, B)).astype(np.int32))
    random_fill(src, lens, 5)
    new_caps = lens + r.integers(0, 5, size=(L, B)).astype(np.int32)      # some streams exactly full
    print(f"case repack dtype={dtype} d={d} Hkv={Hkv} L={L} B={B}", flush=True)
    dst = xkv.XkvCache(L, B, Hkv * 2, Hkv, d, dtype, new_caps)            # zero-filled arenas
    xkv.xkv_repack(src, dst, 0, L)
    torch.cuda.synchronize()
    _check_copy(src, dst)
    dst2 = src.resized(new_caps)                                           # the same into uninitialised arenas
    torch.cuda.synchronize()
    _check_copy(src, dst2, zeroed=False)


def test_repack_layer_range_and_errors(xkv):
    lens = np.array([[300, 10], [70, 513]], np.int32)
    src = xkv.XkvCache(2, 2, 4, 2, 128, "bf16", lens + 4)
    random_fill(src, lens, 8)
    dst = xkv.XkvCache(2, 2, 4, 2, 128, "bf16", lens + 1)
    xkv.xkv_repack(src, dst, 1, 2)
    torch.cuda.synchronize()
    assert list(dst.len) == [0, 0, 70, 513]
    xkv.xkv_repack(src, dst, 0, 1)
    torch.cuda.synchronize()
    _check_copy(src, dst)
    small = xkv.XkvCache(2, 2, 4, 2, 128, "bf16", np.array([[300, 10], [70, 512]], np.int32))
    with pytest.raises(xkv.XkvError) as e:
        xkv.xkv_repack(src, small, 0, 2)
    assert e.value.status == -3 and not small.len.any()           # CAPACITY, nothing done
    other = xkv.XkvCache(2, 2, 8, 2, 128, "bf16", lens + 4)
    with pytest.raises(xkv.XkvError) as e:
        xkv.xkv_repack(src, other, 0, 2)
    assert e.value.status == -1                                    # shapes differ
    with pytest.raises(xkv.XkvError) as e:
        xkv.xkv_repack(src, src, 0, 2)
    assert e.value.status == -1                                    # not in place
