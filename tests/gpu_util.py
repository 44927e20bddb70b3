"""Helpers for the GPU parity tests: move units between the device cache and
the oracle's NumPy form, and the norm-wise error of the tolerance rule."""
import numpy as np
import torch

import xkv_workloads as wl

TOL = {"f32": 1e-5, "bf16": 2e-2}      # relative, norm-wise per vector (fp32 / bf16 inputs)


def rel_err(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


def storage(t):
    return wl.to_numpy_storage(t)


def random_fill(cache, lens, seed, score_scale=1.0, ties=False):
    """Random K, V, score >= 0 and distinct pos for every live slot."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    cache.len[:] = np.asarray(lens, np.int32).reshape(-1)
    for l in range(cache.n_layers):
        for b in range(cache.batch):
            n = cache.length(l, b)
            for h in range(cache.n_kv_heads):
                s0 = cache.stream_slot(l, b, h)
                if n == 0:
                    continue
                cache.k[s0:s0 + n] = torch.randn((n, cache.head_dim), generator=g).to(cache.torch_dtype).cuda()
                cache.v[s0:s0 + n] = torch.randn((n, cache.head_dim), generator=g).to(cache.torch_dtype).cuda()
                if ties:
                    sc = torch.randint(0, 6, (n,), generator=g).float() * 0.125
                else:
                    sc = torch.rand(n, generator=g) * score_scale
                cache.score[s0:s0 + n] = sc.cuda()
                cache.pos[s0:s0 + n] = torch.randperm(n + 3, generator=g)[:n].int().cuda()


def get_unit(cache, l, b, h, n=None):
    n = cache.length(l, b) if n is None else n
    s0 = cache.stream_slot(l, b, h)
    return (storage(cache.k[s0:s0 + n]), storage(cache.v[s0:s0 + n]),
            cache.score[s0:s0 + n].cpu().numpy().copy(), cache.pos[s0:s0 + n].cpu().numpy().copy())
