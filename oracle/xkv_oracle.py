"""CPU oracle for the XKV decode hot path.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain definition that the HIP library is checked
against.  Nothing in the product path may import it: only the tests, the smoke
check and the CPU-baseline leg of the benchmark do.  It shares no code with the
HIP library and imports nothing from it.

Everything here is NumPy in float64 on one unit at a time.  A *unit* is one
(layer, sequence, KV head): n cached tokens with a K row and a V row of d
channels each, an fp32 importance score and an int32 original position.

What follows which passage of the paper (arXiv 2412.05896):

* ``attend_score``      Eq. 1 (Z = softmax(QK^T/sqrt(d_k)) V) and Eq. 2
                        (W_attn); the score update is the Select + Merge step
                        of Eq. 3 / Alg. 2 steps 2-3 with the decode query as the
                        observation row and "sum" in place of "mean".
* ``pooled_keys``       Alg. 2 step 4 (Pooling) as described with the attention
                        processing module in Sec. 4.1.
* ``evict_compact``     Alg. 2 steps 5-7 (TopK, EvictByIndex on K and V).
* ``window_attention_mass``  Alg. 2 steps 1-3 for the prefill phase: W_attn of the
                        observation window (Eq. 2, causal), Select and Merge as
                        in the attention processing module of Sec. 4.1 (Eq. 3).
* ``window_importance``  the attention score distribution vector of a layer as
                        the mini-prefill hands it to the allocator (Sec. 4.1):
                        masses merged over the KV heads, then pooled.
* ``prefill_select``, ``prefill_evict``  Alg. 2 steps 4-7 on a dense prompt:
                        Pooling over the candidate vector, TopK, EvictByIndex as
                        an ordered gather.
* ``retention_ratio``   Eq. 4 (R_i), as a fraction.
* ``allocate_budgets``  Alg. 1 (one token at a time to the layer with the largest
                        next gain) for the two problems of Eq. 17 and Eq. 18.
* ``cache_importance``   the attention score distribution vector of a layer taken
                        from the decode-time cache itself, for re-running Alg. 1
                        during generation (the dynamic tuning of Sec. 2; same
                        role as the vector of Sec. 4.1): the retained tokens'
                        accumulated masses added over the KV heads by original
                        position.
* ``average_allocations``  Sec. 4.3 (sampling-based overhead reduction): the
                        average of the allocation lists recorded on sampled
                        tasks, as an integer list for the next task.

Parity pins: every function here is pinned by tests that do not go through it
(brute force, closed forms, a library routine, hand-worked cases).  The whole
multi-step decode trajectory has no number printed in the paper to compare
with: "parity unpinned" for the trajectory as a whole, it is pinned only
through its per-step parts.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "as_f64",
    "attend_score",
    "pooled_keys",
    "select_keep",
    "evict_compact",
    "window_attention_mass",
    "window_importance",
    "prefill_select",
    "prefill_evict",
    "cache_importance",
    "retention_ratio",
    "allocate_budgets",
    "average_allocations",
    "OracleUnit",
]


# --------------------------------------------------------------------------
# storage helpers
# --------------------------------------------------------------------------
def as_f64(x: np.ndarray) -> np.ndarray:
    """Exact float64 value of stored elements.

    ``x`` is either an fp32 array or a uint16 array of bfloat16 bit patterns
    (the upper half of the fp32 encoding).  Both conversions are exact.
    """
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if x.dtype == np.float32 or x.dtype == np.float64:
        return x.astype(np.float64)
    raise TypeError(f"unsupported element type {x.dtype}")


# --------------------------------------------------------------------------
# Eq. 1 / Eq. 2 and the score update
# --------------------------------------------------------------------------
def attend_score(q, K, V, score, scale=None):
    """One decode query group against one unit.

    q      [G, d]   queries of the G query heads that share this KV head
    K, V   [n, d]   cached rows, *including* the token appended this step
    score  [n]      fp32 importance so far (0 for the appended token)
    scale           logit scale; default 1/sqrt(d)  (Eq. 1)

    Returns ``out`` [G, d] fp32, ``new_score`` [n] fp32 and the fp64
    probability matrix ``p`` [G, n] (rows sum to 1).  With n = 0 the output is
    zero and there is nothing to score.
    """
    q = as_f64(q)
    K = as_f64(K)
    V = as_f64(V)
    G, d = q.shape
    n = K.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    scale = float(scale)
    out = np.zeros((G, d), dtype=np.float64)
    p = np.zeros((G, n), dtype=np.float64)
    if n == 0:
        return out.astype(np.float32), np.zeros(0, dtype=np.float32), p
    for g in range(G):
        s = scale * (K @ q[g])                # logits  q.K_j / sqrt(d)
        m = np.max(s)
        e = np.exp(s - m)
        p[g] = e / np.sum(e)                  # Eq. 2, one row of W_attn
        out[g] = p[g] @ V                     # Eq. 1
    mass = np.sum(p, axis=0)                  # Merge over the group's rows (sum)
    new_score = (np.asarray(score, dtype=np.float32).astype(np.float64) + mass).astype(np.float32)
    return out.astype(np.float32), new_score, p


# --------------------------------------------------------------------------
# Alg. 2 step 4: pooling
# --------------------------------------------------------------------------
def pooled_keys(score, pool_size: int) -> np.ndarray:
    """Window sum of width ``pool_size`` (odd), stride 1, same length, zeros
    outside the array.  Adds are fp32 and go left to right over the window, so
    the result is defined bit for bit.  (Average pooling times the constant
    window width: the ranking is the same.)
    """
    if pool_size < 1 or pool_size % 2 == 0:
        raise ValueError("pool_size must be odd and >= 1")
    s = np.asarray(score, dtype=np.float32)
    n = s.shape[0]
    h = pool_size // 2
    if h == 0:
        return s.copy()
    padded = np.zeros(n + 2 * h, dtype=np.float32)
    padded[h:h + n] = s
    acc = padded[0:n].copy()                  # term j-h
    for t in range(1, pool_size):             # then j-h+1 ... j+h, in order
        acc = (acc + padded[t:t + n]).astype(np.float32)
    return acc


# --------------------------------------------------------------------------
# Alg. 2 step 5: TopK
# --------------------------------------------------------------------------
def select_keep(score, pos, budget: int, pool_size: int = 1, n_protect: int = 0) -> np.ndarray:
    """Slots kept by the top-``budget`` rule, as a sorted index array.

    Key = pooled score; the ``n_protect`` most recent original positions
    (pos >= 1 + max(pos) - n_protect) are never candidates for eviction, they
    get key +inf.  Order is (key descending, slot ascending); the first
    min(budget, n) slots of that order are kept.
    """
    s = np.asarray(score, dtype=np.float32)
    n = s.shape[0]
    kk = min(int(budget), n)
    if kk <= 0:
        return np.zeros(0, dtype=np.int64)
    key = pooled_keys(s, pool_size)
    if n_protect > 0 and n > 0:
        pos = np.asarray(pos)
        P = 1 + int(np.max(pos))
        key = key.copy()
        key[pos >= P - n_protect] = np.inf
    order = np.argsort(-key.astype(np.float64), kind="stable")
    return np.sort(order[:kk])


# --------------------------------------------------------------------------
# Alg. 2 steps 5-7: TopK + EvictByIndex, in place by hole filling
# --------------------------------------------------------------------------
def evict_compact(K, V, score, pos, budget: int, pool_size: int = 1, n_protect: int = 0):
    """Keep the top-``budget`` tokens of a unit and compact it.

    The kept tokens that sit at slots >= k' (k' = min(budget, n)) are moved,
    in ascending slot order, into the evicted slots < k', in ascending slot
    order.  Everything else stays where it is.  Returns the new
    (K, V, score, pos), each of length k', and ``kept_idx`` [k'] = the slot
    each final slot's content came from.
    """
    K = np.asarray(K)
    V = np.asarray(V)
    score = np.asarray(score, dtype=np.float32)
    pos = np.asarray(pos, dtype=np.int32)
    n = score.shape[0]
    kk = min(int(budget), n)
    keep = select_keep(score, pos, budget, pool_size, n_protect)
    kept = np.zeros(n, dtype=bool)
    kept[keep] = True
    holes = [s for s in range(kk) if not kept[s]]
    movers = [s for s in range(kk, n) if kept[s]]
    assert len(holes) == len(movers)
    kept_idx = np.arange(kk, dtype=np.int32)
    for hslot, mslot in zip(holes, movers):
        kept_idx[hslot] = mslot
    return (K[kept_idx].copy(), V[kept_idx].copy(), score[kept_idx].copy(),
            pos[kept_idx].copy(), kept_idx)


# --------------------------------------------------------------------------
# Alg. 2 as written, for the prefill phase (Sec. 4.1, attention processing)
# --------------------------------------------------------------------------
def window_row_lse(q_win, K, scale=None) -> np.ndarray:
    """Natural logarithm of the softmax normaliser (Eq. 2) of every window row.

    q_win [G, ows, d], K [t, d] as for ``window_attention_mass``.  Returns
    lse [G, ows] in float64 with
    lse[g][r] = ln sum_{j <= t - ows + r} exp(scale * q_win[g][r] . K[j]):
    what an attention forward pass over the prompt leaves behind for its last
    ows query rows, so that W_attn[g][t - ows + r][j] = exp(logit - lse[g][r]).
    """
    q_win = as_f64(q_win)
    K = as_f64(K)
    G, ows, d = q_win.shape
    t = K.shape[0]
    if ows < 1 or ows > t:
        raise ValueError("need 1 <= ows <= t")
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    scale = float(scale)
    lse = np.zeros((G, ows), dtype=np.float64)
    for g in range(G):
        for r in range(ows):
            last = t - ows + r
            s = scale * (K[:last + 1] @ q_win[g, r])
            top = np.max(s)
            lse[g, r] = top + np.log(np.sum(np.exp(s - top)))
    return lse


def window_attention_mass(q_win, K, scale=None, lse=None) -> np.ndarray:
    """Attention mass that the observation window puts on every prompt token.

    q_win  [G, ows, d]  queries of the last ``ows`` prompt positions, for the G
                        query heads that share this KV head
    K      [t, d]       keys of the whole prompt (t >= ows)

    Window row r is prompt position t - ows + r and, the attention being
    causal, sees positions 0 .. t - ows + r; its softmax (Eq. 2) runs over
    exactly those.  Returns w [t] in float64 with
    w[j] = sum over g and r of W_attn[g][t - ows + r][j].  Its first t - ows
    entries are the Select block merged over the window rows and the heads
    (sum; the paper's mean is this divided by the constant ows); the last ows
    entries are the mass the window puts on itself.  sum(w) = G * ows.

    lse [G, ows] (optional): the rows' normalisers as the caller has them
    (``window_row_lse``); the weights are then exp(logit - lse[g][r]), whatever
    lse holds, and the softmax is not normalised again.
    """
    q_win = as_f64(q_win)
    K = as_f64(K)
    G, ows, d = q_win.shape
    t = K.shape[0]
    if ows < 1 or ows > t:
        raise ValueError("need 1 <= ows <= t")
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    scale = float(scale)
    if lse is not None:
        lse = as_f64(lse)
        if lse.shape != (G, ows):
            raise ValueError("lse must be [G, ows]")
    w = np.zeros(t, dtype=np.float64)
    for g in range(G):
        for r in range(ows):
            last = t - ows + r                # the row's own position
            s = scale * (K[:last + 1] @ q_win[g, r])
            if lse is None:
                e = np.exp(s - np.max(s))
                w[:last + 1] += e / np.sum(e)
            else:
                w[:last + 1] += np.exp(s - lse[g, r])
    return w


def window_importance(q_win, K, pool_size: int = 1, scale=None) -> np.ndarray:
    """Attention score distribution vector of one (layer, sequence).

    q_win [Hkv, G, ows, d], K [Hkv, t, d].  The candidates' masses
    (``window_attention_mass``, first t - ows entries) are added over the KV
    heads, then pooled: window sum of width ``pool_size``, stride 1, zeros
    outside the candidate vector.  float64 throughout; no decision is taken
    here, so nothing needs a fixed precision.
    """
    q_win = np.asarray(q_win)
    K = np.asarray(K)
    Hkv, G, ows, d = q_win.shape
    t = K.shape[1]
    tc = t - ows
    total = np.zeros(tc, dtype=np.float64)
    for h in range(Hkv):
        total += window_attention_mass(q_win[h], K[h], scale)[:tc]
    half = pool_size // 2
    if pool_size < 1 or pool_size % 2 == 0:
        raise ValueError("pool_size must be odd and >= 1")
    out = np.zeros(tc, dtype=np.float64)
    for j in range(tc):
        lo, hi = max(0, j - half), min(tc, j + half + 1)
        out[j] = np.sum(total[lo:hi])
    return out


def prefill_select(w, ows: int, budget: int, pool_size: int = 1) -> np.ndarray:
    """Prompt positions kept by Alg. 2 steps 4-5, ascending.

    w [t] is the fp32 mass vector.  The candidates are the first t - ows
    positions; their keys are the pooled candidate vector (``pooled_keys`` of
    w[:t - ows]: nothing of the window enters a key).  The window's ows
    positions are always kept and count towards the budget, so
    min(budget, t) - ows candidates are kept: the largest keys, equal keys by
    lower position.
    """
    w = np.asarray(w, dtype=np.float32)
    t = w.shape[0]
    kk = min(int(budget), t)
    if kk < ows:
        raise ValueError("the budget must cover the observation window")
    tc = t - ows
    key = pooled_keys(w[:tc], pool_size)
    order = np.argsort(-key.astype(np.float64), kind="stable")
    cand = np.sort(order[:kk - ows])
    return np.concatenate([cand, np.arange(tc, t)]).astype(np.int64)


def prefill_evict(q_win, K, V, budget: int, ows: int, pool_size: int = 1, scale=None, w=None):
    """Alg. 2 on one unit of a dense prompt.

    Returns (K', V', score', pos', w): the kept tokens in ascending position
    order, score' = their fp32 mass (not pooled), pos' = their positions, and
    the fp32 mass vector the selection was taken on.  If ``w`` is given (fp32),
    the selection uses it instead of this function's own: a decision that
    floating point takes must be taken on the same bits by both sides of a
    parity test.
    """
    K = np.asarray(K)
    V = np.asarray(V)
    if w is None:
        w = window_attention_mass(q_win, K, scale).astype(np.float32)
    w = np.asarray(w, dtype=np.float32)
    keep = prefill_select(w, ows, budget, pool_size)
    return K[keep].copy(), V[keep].copy(), w[keep].copy(), keep.astype(np.int32), w


# --------------------------------------------------------------------------
# Score vector of a layer from the decode-time cache (input of Alg. 1)
# --------------------------------------------------------------------------
def cache_importance(pos_per_head, score_per_head, n_pos: int) -> np.ndarray:
    """Position-indexed score vector of one (layer, sequence).

    pos_per_head[h], score_per_head[h]  original positions (distinct within a
    head) and fp32 accumulated masses of the tokens that KV head h still holds,
    in any order.  After per-head eviction the heads hold different tokens, so
    the vector is indexed by original position:

        w[p] = sum over the heads h that still hold position p of its score,

    added in head order in fp32 (so that the result is defined bit for bit: it
    decides an integer allocation); a position no head holds has w = 0, and
    tokens whose position lies outside [0, n_pos) are left out.  Before any
    eviction this is the head-merged vector of the attention processing module
    (Sec. 4.1) with a sum as the merge.
    """
    w = np.zeros(int(n_pos), dtype=np.float32)
    for pos, score in zip(pos_per_head, score_per_head):
        pos = np.asarray(pos, dtype=np.int64)
        score = np.asarray(score, dtype=np.float32)
        if pos.shape != score.shape:
            raise ValueError("one score per position")
        inside = (pos >= 0) & (pos < n_pos)
        if np.unique(pos[inside]).size != int(inside.sum()):
            raise ValueError("positions of a head must be distinct")
        w[pos[inside]] = (w[pos[inside]] + score[inside]).astype(np.float32)
    return w


# --------------------------------------------------------------------------
# Eq. 4
# --------------------------------------------------------------------------
def retention_ratio(w, n: int) -> float:
    """R = Sum(TopK(n, w)) / Sum(w) as a fraction in [0, 1]."""
    w = np.asarray(w, dtype=np.float64)
    tot = float(np.sum(w))
    if tot == 0.0:
        return 0.0
    top = np.sort(w)[::-1][:max(int(n), 0)]
    return float(np.sum(top) / tot)


# --------------------------------------------------------------------------
# Alg. 1
# --------------------------------------------------------------------------
def _normalised_gains(w):
    """Per layer: gain[r] = (r+1)-th largest value / the layer's sum, float64.

    gain[r] is what L * R_avg grows by when the layer goes from r to r + 1
    tokens (Eq. 21).  The sum is taken in float64 over the values in ascending
    order, one after the other, so its value does not depend on who computes
    it; a layer whose values sum to zero gains nothing from any token.
    """
    gains = []
    for w_l in w:
        a = np.asarray(w_l, dtype=np.float32)
        if a.ndim != 1:
            raise ValueError("each w_l must be a vector")
        if not np.all(np.isfinite(a)) or np.any(a < 0):
            raise ValueError("w must be finite and non-negative")
        asc = np.sort(a).astype(np.float64)
        total = float(np.add.accumulate(asc)[-1]) if asc.size else 0.0
        desc = asc[::-1]
        gains.append(desc / total if total != 0.0 else np.zeros_like(desc))
    return gains


def allocate_budgets(w, total_size=None, target_ravg=None, min_budget=None, max_budget=None):
    """Greedy solver of the two allocation problems (Alg. 1; Eq. 17, Eq. 18).

    w            list of L vectors (any order, non-negative)
    total_size   N of Eq. 17: hand out tokens until sum(n_l) = N
    target_ravg  set value of Eq. 18, a fraction: hand out tokens until
                 R_avg >= it; exactly one of the two is given
    min_budget / max_budget  optional per-layer floors and caps

    Every layer keeps a cursor n_l into its gains sorted in descending order.
    One token at a time goes to the layer whose next gain (Eq. 21) is the
    largest over all layers, the lowest layer index among equals; a layer at its
    cap no longer takes part.  Returns (budgets int64 [L], R_avg fraction).
    """
    if (total_size is None) == (target_ravg is None):
        raise ValueError("give exactly one of total_size / target_ravg")
    gains = _normalised_gains(w)
    L = len(gains)
    floor = [0] * L if min_budget is None else [int(x) for x in min_budget]
    cap = [g.size for g in gains] if max_budget is None else \
        [min(int(x), g.size) for x, g in zip(max_budget, gains)]
    if any(floor[l] < 0 or floor[l] > cap[l] for l in range(L)):
        raise ValueError("infeasible: floor above cap")

    n = list(floor)
    held = 0.0                                # L * R_avg of the current sizes
    for l in range(L):
        for r in range(n[l]):
            held += gains[l][r]
    nxt = np.array([gains[l][n[l]] if n[l] < cap[l] else -np.inf for l in range(L)], dtype=np.float64)

    def give_one():
        nonlocal held
        l = int(np.argmax(nxt))               # first index of the maximum
        held += nxt[l]
        n[l] += 1
        nxt[l] = gains[l][n[l]] if n[l] < cap[l] else -np.inf

    if total_size is not None:
        N = int(total_size)
        if N < sum(floor) or N > sum(cap):
            raise ValueError("infeasible total size")
        for _ in range(N - sum(floor)):
            give_one()
    else:
        target = float(target_ravg)
        while held / L < target and np.max(nxt) > -np.inf:
            give_one()

    ravg = sum(float(np.sum(gains[l][:n[l]])) for l in range(L) if n[l] > 0) / L
    return np.asarray(n, dtype=np.int64), ravg


# --------------------------------------------------------------------------
# Sec. 4.3: averaged allocation list of sampled tasks
# --------------------------------------------------------------------------
def average_allocations(lists, total_size: int, min_budget=None, max_budget=None) -> np.ndarray:
    """Allocation list for a new task from the lists recorded on sampled tasks.

    lists [n_samples, L] non-negative integers.  The per-layer averages are
    scaled so that they sum to ``total_size`` (they already do when every
    sample was allocated that total), x_l = total_size * sum_s lists[s][l] /
    sum of all entries, in exact rational arithmetic.  Rounding is by largest
    remainder: every layer gets floor(x_l), the layers with the largest
    fractional parts one more until the total is met (equal parts: lower layer
    first).  With bounds the list is then clamped, and single tokens are added
    to the layer furthest below its x_l (below its cap), or taken from the one
    furthest above (above its floor), until the total is met again.
    """
    from fractions import Fraction
    lists = np.asarray(lists, dtype=np.int64)
    if lists.ndim != 2 or lists.shape[0] < 1 or np.any(lists < 0):
        raise ValueError("lists must be [n_samples, L] non-negative")
    L = lists.shape[1]
    col = [int(v) for v in lists.sum(axis=0)]
    tot = sum(col)
    N = int(total_size)
    lo = [0] * L if min_budget is None else [int(v) for v in min_budget]
    hi = [None] * L if max_budget is None else [int(v) for v in max_budget]
    if tot == 0:
        raise ValueError("the samples hold no tokens")
    if any(h is not None and l > h for l, h in zip(lo, hi)) or N < sum(lo) or \
            (all(h is not None for h in hi) and N > sum(hi)):
        raise ValueError("infeasible")
    x = [Fraction(c * N, tot) for c in col]
    n = [int(v) for v in (f.numerator // f.denominator for f in x)]
    frac = [x[l] - n[l] for l in range(L)]
    for l in sorted(range(L), key=lambda l: (-frac[l], l))[:N - sum(n)]:
        n[l] += 1
    n = [max(lo[l], n[l] if hi[l] is None else min(hi[l], n[l])) for l in range(L)]
    while sum(n) < N:
        cand = [l for l in range(L) if hi[l] is None or n[l] < hi[l]]
        l = min(cand, key=lambda l: (-(x[l] - n[l]), l))
        n[l] += 1
    while sum(n) > N:
        cand = [l for l in range(L) if n[l] > lo[l]]
        l = min(cand, key=lambda l: (-(n[l] - x[l]), l))
        n[l] -= 1
    return np.asarray(n, dtype=np.int64)


# --------------------------------------------------------------------------
# a unit with state, for multi-step runs
# --------------------------------------------------------------------------
class OracleUnit:
    """State of one (layer, sequence, KV head) across decode steps."""

    def __init__(self, K, V, score=None, pos=None):
        self.K = np.array(K, copy=True)
        self.V = np.array(V, copy=True)
        n = self.K.shape[0]
        self.score = np.zeros(n, np.float32) if score is None else np.array(score, np.float32)
        self.pos = np.arange(n, dtype=np.int32) if pos is None else np.array(pos, np.int32)

    @property
    def n(self):
        return self.K.shape[0]

    def append(self, k_new, v_new, pos_new):
        """The new token's K/V row joins the cache with score 0 (Sec. 4.1,
        generation phase)."""
        self.K = np.concatenate([self.K, np.asarray(k_new).reshape(1, -1)], axis=0)
        self.V = np.concatenate([self.V, np.asarray(v_new).reshape(1, -1)], axis=0)
        self.score = np.concatenate([self.score, np.zeros(1, np.float32)])
        self.pos = np.concatenate([self.pos, np.asarray([pos_new], np.int32)])

    def attend(self, q, scale=None):
        out, self.score, p = attend_score(q, self.K, self.V, self.score, scale)
        return out, p

    def evict(self, budget, pool_size=1, n_protect=0):
        self.K, self.V, self.score, self.pos, kept_idx = evict_compact(
            self.K, self.V, self.score, self.pos, budget, pool_size, n_protect)
        return kept_idx
