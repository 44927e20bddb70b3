"""Pins for the oracle's attention + scoring (Eq. 1, Eq. 2, Select/Merge of
Eq. 3): none of them goes through the oracle's own formula."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import xkv_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand(n, d, G, seed):
    r = np.random.default_rng(seed)
    return (r.standard_normal((G, d)).astype(np.float32),
            r.standard_normal((n, d)).astype(np.float32),
            r.standard_normal((n, d)).astype(np.float32))


def test_hand_example_from_golden():
    vals = {}
    for line in open(os.path.join(GOLD, "attention_hand_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        vals[k] = np.array([float(x) for x in v])
    K = np.array([[math.sqrt(2.0) * math.log(3.0), 7.0], [0.0, -5.0]], np.float64)
    V = np.array([[4.0, 0.0], [0.0, 8.0]], np.float64)
    q = np.array([[1.0, 0.0], [0.0, 0.0]], np.float64)
    out, score, p = orc.attend_score(q, K, V, np.zeros(2, np.float32))
    np.testing.assert_allclose(p[0], vals["p"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(p[1], vals["p2"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(out[0], vals["z"], rtol=0, atol=1e-6)
    np.testing.assert_allclose(out[1], vals["z2"], rtol=0, atol=1e-6)
    np.testing.assert_allclose(score, vals["mass"], rtol=0, atol=1e-7)


def test_brute_force_python_loops():
    """Scalar loops with math.exp on a tiny case."""
    q, K, V = _rand(5, 3, 2, 0)
    sc0 = np.array([0.5, 0.0, 1.25, 0.0, 2.0], np.float32)
    out, score, p = orc.attend_score(q, K, V, sc0)
    for g in range(2):
        logit = [sum(float(q[g, c]) * float(K[j, c]) for c in range(3)) / math.sqrt(3.0) for j in range(5)]
        mx = max(logit)
        ex = [math.exp(x - mx) for x in logit]
        tot = sum(ex)
        for j in range(5):
            assert abs(p[g, j] - ex[j] / tot) < 1e-15
        for c in range(3):
            z = sum(ex[j] / tot * float(V[j, c]) for j in range(5))
            assert abs(out[g, c] - z) < 1e-6
    for j in range(5):
        assert abs(score[j] - (float(sc0[j]) + p[0, j] + p[1, j])) < 1e-6


@pytest.mark.parametrize("n,d,G", [(1, 64, 1), (37, 64, 4), (300, 128, 8)])
def test_matches_library_sdpa_float64(n, d, G):
    """With nothing evicted the path is plain attention with a one-row query:
    torch's scaled_dot_product_attention on CPU in float64."""
    q, K, V = _rand(n, d, G, 1)
    out, _, _ = orc.attend_score(q, K, V, np.zeros(n, np.float32))
    tq = torch.from_numpy(q).double()[None, :, None, :]          # [1, G, 1, d]
    tk = torch.from_numpy(K).double()[None, None].expand(1, G, n, d)
    tv = torch.from_numpy(V).double()[None, None].expand(1, G, n, d)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0, :].numpy()
    np.testing.assert_allclose(out, ref, rtol=0, atol=2e-6)


def test_dense_matrix_route_and_custom_scale():
    """Materialise the dense G x n probability matrix a different way
    (log-sum-exp through torch) and multiply."""
    q, K, V = _rand(129, 64, 4, 2)
    scale = 0.37
    out, score, p = orc.attend_score(q, K, V, np.zeros(129, np.float32), scale=scale)
    logits = torch.from_numpy(q).double() @ torch.from_numpy(K).double().T * scale
    P = torch.exp(logits - torch.logsumexp(logits, dim=1, keepdim=True))
    np.testing.assert_allclose(p, P.numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(out, (P @ torch.from_numpy(V).double()).numpy(), rtol=0, atol=2e-6)
    np.testing.assert_allclose(score, P.sum(0).numpy(), rtol=0, atol=1e-6)


def test_closed_forms():
    r = np.random.default_rng(3)
    n, d = 50, 64
    V = r.standard_normal((n, d)).astype(np.float32)
    q = r.standard_normal((1, d)).astype(np.float32)
    # all keys equal -> uniform weights, output = mean of V
    K = np.tile(r.standard_normal((1, d)).astype(np.float32), (n, 1))
    out, score, p = orc.attend_score(q, K, V, np.zeros(n, np.float32))
    np.testing.assert_allclose(p[0], np.full(n, 1.0 / n), atol=1e-15)
    np.testing.assert_allclose(out[0], V.astype(np.float64).mean(0), atol=1e-6)
    # one key dominates -> output tends to that value row
    K = r.standard_normal((n, d)).astype(np.float32)
    K[17] = 100.0 * q[0]
    out, score, p = orc.attend_score(q, K, V, np.zeros(n, np.float32))
    assert p[0, 17] > 1 - 1e-12
    np.testing.assert_allclose(out[0], V[17], atol=1e-6)
    # constant V -> constant output whatever the weights
    Vc = np.tile(np.arange(d, dtype=np.float32), (n, 1))
    out, _, _ = orc.attend_score(q, K, Vc, np.zeros(n, np.float32))
    np.testing.assert_allclose(out[0], np.arange(d), atol=1e-5)


def test_rows_sum_to_one_and_invariances():
    q, K, V = _rand(257, 64, 4, 4)
    out, score, p = orc.attend_score(q, K, V, np.zeros(257, np.float32))
    assert np.all(np.abs(p.sum(1) - 1.0) <= 1e-12)
    assert abs(float(score.astype(np.float64).sum()) - 4.0) < 1e-5
    # adding the same vector u to every key shifts all logits of a head by q.u
    u = np.random.default_rng(5).standard_normal(64).astype(np.float32)
    K2 = (K.astype(np.float64) + u.astype(np.float64))
    _, _, p2 = orc.attend_score(q.astype(np.float64), K2, V.astype(np.float64), np.zeros(257, np.float32))
    np.testing.assert_allclose(p2, p, atol=1e-12)
    # permuting the slots permutes probabilities and scores, leaves outputs
    perm = np.random.default_rng(6).permutation(257)
    out3, score3, p3 = orc.attend_score(q, K[perm], V[perm], np.zeros(257, np.float32))
    np.testing.assert_allclose(p3, p[:, perm], atol=1e-15)
    np.testing.assert_allclose(out3, out, atol=1e-6)
    np.testing.assert_array_equal(score3, score[perm])


def test_mass_conservation_over_steps_with_eviction():
    """Retained score + evicted score = G * (queries so far), per unit."""
    r = np.random.default_rng(7)
    G, d, n0, budget = 2, 64, 40, 24
    u = orc.OracleUnit(r.standard_normal((n0, d)).astype(np.float32),
                       r.standard_normal((n0, d)).astype(np.float32))
    evicted_mass = 0.0
    for step in range(12):
        u.append(r.standard_normal(d).astype(np.float32), r.standard_normal(d).astype(np.float32), n0 + step)
        u.attend(r.standard_normal((G, d)).astype(np.float32))
        before = float(u.score.astype(np.float64).sum())
        if step >= 3:
            u.evict(budget)
            assert u.n == budget
        evicted_mass += before - float(u.score.astype(np.float64).sum())
        total = float(u.score.astype(np.float64).sum()) + evicted_mass
        assert abs(total - G * (step + 1)) < 1e-4


def test_empty_unit():
    out, score, p = orc.attend_score(np.ones((2, 8), np.float32), np.zeros((0, 8), np.float32),
                                     np.zeros((0, 8), np.float32), np.zeros(0, np.float32))
    assert out.shape == (2, 8) and not out.any() and score.shape == (0,)


def test_bf16_bits_are_read_exactly():
    t = torch.randn(1000, generator=torch.Generator().manual_seed(0)).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(orc.as_f64(bits), t.double().numpy())
    # and a bf16 unit gives the same result as its fp32-widened copy
    r = np.random.default_rng(8)
    K = torch.from_numpy(r.standard_normal((33, 64)).astype(np.float32)).to(torch.bfloat16)
    V = torch.from_numpy(r.standard_normal((33, 64)).astype(np.float32)).to(torch.bfloat16)
    q = torch.from_numpy(r.standard_normal((1, 64)).astype(np.float32)).to(torch.bfloat16)
    b = lambda x: x.view(torch.int16).numpy().view(np.uint16)
    o1, s1, _ = orc.attend_score(b(q), b(K), b(V), np.zeros(33, np.float32))
    o2, s2, _ = orc.attend_score(q.float().numpy(), K.float().numpy(), V.float().numpy(), np.zeros(33, np.float32))
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(s1, s2)
