"""Seeded synthetic workloads for the XKV decode hot path.

Input generation only: shapes, sizes, random values and the ragged layout
tables.  None of the method's arithmetic (attention, scoring, selection,
allocation) lives here, so the tests, the benchmark, the HIP binding's callers
and the CPU oracle's callers can all draw the same inputs from it.

The paper's own workloads are long prompts pushed through a language model;
neither is available offline, so these stand in for them: attention geometry of
the named model family, N(0,1) keys/values/queries, and a few "heavy hitter"
cached tokens whose keys have a larger norm, which gives the sparse,
few-dominant-tokens importance profile the paper describes for real prompts
(Sec. 3.1, discussion of the attention-score heat map).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

SEED_BASE = 1234


@dataclass(frozen=True)
class Workload:
    name: str
    index: int              # position in the benchmark's configuration list
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str              # "f32" | "bf16"
    batch: int
    context: int            # prompt tokens in the cache before the first decode step
    decode_steps: int
    budget_frac: Optional[float] = None      # total budget / (L * context)
    fixed_budgets: Optional[tuple] = None    # per-layer budgets given outright
    min_budget: int = 0
    heavy: dict = field(default_factory=dict)  # heavy-hitter recipe
    budget_rule: str = "allocator"           # "fixed" | "allocator" | "dirichlet"

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    @property
    def total_budget(self) -> int:
        if self.fixed_budgets is not None:
            return int(sum(self.fixed_budgets))
        return int(math.floor(self.budget_frac * self.n_layers * self.context + 1e-9))

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


WORKLOADS = {
    "tiny_f32": Workload("tiny_f32", 0, 4, 4, 4, 64, "f32", 1, 512, 16,
                         fixed_budgets=(384, 256, 128, 64), budget_rule="fixed",
                         heavy={"sinks": 4, "sink_scale": 4.0}),
    "llama2_7b_4k": Workload("llama2_7b_4k", 1, 32, 32, 32, 128, "bf16", 1, 4096, 64,
                             budget_frac=0.40, heavy={"frac": 0.01, "scale": 3.0}),
    "llama2_7b_32k": Workload("llama2_7b_32k", 2, 32, 32, 32, 128, "bf16", 1, 32768, 128,
                              budget_frac=0.20, heavy={"frac": 0.01, "scale": 3.0}),
    "mistral_7b_gqa_b32": Workload("mistral_7b_gqa_b32", 3, 32, 32, 8, 128, "bf16", 32, 16384, 64,
                                   budget_frac=0.30, budget_rule="dirichlet",
                                   heavy={"count": 64, "scale": 3.0, "per_sequence": True}),
    "llama3_70b_128k": Workload("llama3_70b_128k", 4, 80, 64, 8, 128, "bf16", 4, 131072, 32,
                                budget_frac=0.15, min_budget=256,
                                heavy={"sinks": 4, "sink_scale": 4.0, "frac": 0.005, "scale": 3.0}),
}


def scaled(w: Workload, **changes) -> Workload:
    """A copy of a workload with some fields changed (reduced test sizes)."""
    d = {f: getattr(w, f) for f in w.__dataclass_fields__}
    d.update(changes)
    return Workload(**d)


def _rng(seed: int, stream: str) -> np.random.Generator:
    """Independent sub-stream per tensor name."""
    tag = int.from_bytes(stream.encode()[:8].ljust(8, b"\0"), "little")
    return np.random.default_rng([seed, tag])


# --------------------------------------------------------------------------
# per-layer importance curves for the allocator
# --------------------------------------------------------------------------
def zipf_importance_curves(n_layers: int, length: int, seed: int) -> List[np.ndarray]:
    """Layer l gets w_l[j] = (rank_l(j) + 1) ** (-s_l) as fp32, with the Zipf
    exponent s_l uniform in [0.6, 1.4) and rank_l a random permutation: each
    layer has its own concentration, the layer-to-layer difference the paper
    calls DDID."""
    r = _rng(seed, "zipf")
    out = []
    for _ in range(n_layers):
        s = 0.6 + 0.8 * r.random()
        perm = r.permutation(length)
        out.append(np.power(perm.astype(np.float64) + 1.0, -s).astype(np.float32))
    return out


def dirichlet_budgets(n_layers: int, batch: int, context: int, total: int, seed: int,
                      floor: int = 64) -> np.ndarray:
    """Per-sequence random per-layer budgets that sum to ``total`` exactly:
    floor + largest-remainder rounding of (total - L*floor) * Dirichlet(1),
    clamped to the context length with the excess handed to the other layers.
    Returns int32 [n_layers, batch]."""
    r = _rng(seed, "dirichlet")
    out = np.zeros((n_layers, batch), dtype=np.int32)
    for b in range(batch):
        u = r.dirichlet(np.ones(n_layers))
        spare = total - n_layers * floor
        raw = spare * u
        base = np.floor(raw).astype(np.int64)
        rem = spare - int(base.sum())
        order = np.argsort(-(raw - base), kind="stable")
        base[order[:rem]] += 1
        bud = base + floor
        while True:                           # clamp and redistribute
            over = np.maximum(bud - context, 0)
            excess = int(over.sum())
            if excess == 0:
                break
            bud = np.minimum(bud, context)
            room = np.flatnonzero(bud < context)
            share, extra = divmod(excess, room.size)
            bud[room] += share
            bud[room[:extra]] += 1
        assert int(bud.sum()) == total
        out[:, b] = bud
    return out


# --------------------------------------------------------------------------
# ragged layout
# --------------------------------------------------------------------------
def region_table(caps: np.ndarray, n_kv_heads: int):
    """caps int [L, B] -> (region_off int64 [L*B], cap int32 [L*B], arena_slots).
    Region (l, b) holds n_kv_heads streams of cap[l, b] slots each."""
    cap = np.ascontiguousarray(caps, dtype=np.int32).reshape(-1)
    sizes = cap.astype(np.int64) * n_kv_heads
    off = np.zeros_like(sizes)
    if sizes.size > 1:
        off[1:] = np.cumsum(sizes)[:-1]
    return off, cap, int(sizes.sum())


def round_up(x, m):
    return (np.asarray(x) + m - 1) // m * m


# --------------------------------------------------------------------------
# cache contents
# --------------------------------------------------------------------------
def heavy_positions(w: Workload, b: int) -> dict:
    """position -> key scale for sequence b (the same for all layers, heads)."""
    h = w.heavy
    out = {}
    r = _rng(w.seed, f"hv{b if h.get('per_sequence') else 0}")
    if "frac" in h:
        cnt = max(1, int(round(h["frac"] * w.context)))
        for p in r.choice(w.context, size=cnt, replace=False):
            out[int(p)] = float(h["scale"])
    if "count" in h:
        for p in r.choice(w.context, size=min(h["count"], w.context), replace=False):
            out[int(p)] = float(h["scale"])
    for p in range(min(h.get("sinks", 0), w.context)):
        out[p] = float(h["sink_scale"])
    return out


def fill_prompt_cache(w: Workload, k_arena: torch.Tensor, v_arena: torch.Tensor,
                      score: torch.Tensor, pos: torch.Tensor,
                      region_off: np.ndarray, cap: np.ndarray) -> None:
    """Write the step-0 state: ``context`` tokens per stream, K, V ~ N(0,1)
    rounded to the storage type, heavy-hitter keys scaled, score 0, pos 0..T-1.
    Arenas are [arena_slots, d] (k, v) and [arena_slots] (score, pos)."""
    dev = k_arena.device
    T, Hkv, d = w.context, w.n_kv_heads, w.head_dim
    if dev.type == "cpu" or w.n_layers * w.batch * Hkv * T * d <= (1 << 26):
        # small caches come from the CPU generator: bit-reproducible anywhere
        g = torch.Generator(device="cpu")
        g.manual_seed(w.seed)
        # one bit-reproducible draw per tensor, [L, B, Hkv, T, d]
        kk = torch.randn((w.n_layers, w.batch, Hkv, T, d), generator=g, dtype=torch.float32)
        vv = torch.randn((w.n_layers, w.batch, Hkv, T, d), generator=g, dtype=torch.float32)
        for l in range(w.n_layers):
            for b in range(w.batch):
                i = l * w.batch + b
                for h in range(Hkv):
                    s0 = int(region_off[i]) + h * int(cap[i])
                    k_arena[s0:s0 + T] = kk[l, b, h].to(k_arena.dtype).to(dev)
                    v_arena[s0:s0 + T] = vv[l, b, h].to(v_arena.dtype).to(dev)
    else:
        g = torch.Generator(device=dev)
        g.manual_seed(w.seed)
        k_arena.normal_(generator=g)
        v_arena.normal_(generator=g)
    score.zero_()
    ar = torch.arange(T, dtype=torch.int32, device=dev)
    for b in range(w.batch):
        hv = heavy_positions(w, b)
        hp = torch.tensor(sorted(hv), dtype=torch.int64, device=dev)
        hs = torch.tensor([hv[p] for p in sorted(hv)], dtype=torch.float32, device=dev)
        for l in range(w.n_layers):
            i = l * w.batch + b
            for h in range(Hkv):
                s0 = int(region_off[i]) + h * int(cap[i])
                pos[s0:s0 + T] = ar
                if hp.numel():
                    rows = k_arena[s0 + hp].to(torch.float32) * hs[:, None]
                    k_arena[s0 + hp] = rows.to(k_arena.dtype)


def dense_prompt_layer(w: Workload, layer: int, ows: int, device="cpu"):
    """One layer of a dense prompt for the prefill-phase eviction: k_src, v_src
    [1, B, Hkv, T, d] ~ N(0,1) in the storage type with the workload's
    heavy-hitter keys scaled, and q_win [1, B, Hq, ows, d] ~ N(0,1)."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed + 104729 * (layer + 1))
    T, d = w.context, w.head_dim
    k = torch.randn((1, w.batch, w.n_kv_heads, T, d), generator=g, dtype=torch.float32, device=dev)
    for b in range(w.batch):
        hp = heavy_positions(w, b)
        if hp:
            idx = torch.tensor(sorted(hp), dtype=torch.long, device=dev)
            sc = torch.tensor([hp[p] for p in sorted(hp)], dtype=torch.float32, device=dev)
            k[0, b, :, idx, :] *= sc[None, :, None]
    k = k.to(w.torch_dtype())
    v = torch.randn((1, w.batch, w.n_kv_heads, T, d), generator=g, dtype=torch.float32, device=dev).to(w.torch_dtype())
    q = torch.randn((1, w.batch, w.n_q_heads, ows, d), generator=g, dtype=torch.float32, device=dev).to(w.torch_dtype())
    return q, k, v


def decode_inputs(w: Workload, steps: Optional[int] = None, device="cpu"):
    """q [steps, L, B, Hq, d], k_new and v_new [steps, L, B, Hkv, d] ~ N(0,1) in
    the storage type, and pos_new int32 [steps, B] = context + step."""
    steps = w.decode_steps if steps is None else steps
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed + 7919)
    shp_q = (steps, w.n_layers, w.batch, w.n_q_heads, w.head_dim)
    shp_k = (steps, w.n_layers, w.batch, w.n_kv_heads, w.head_dim)
    q = torch.randn(shp_q, generator=g, dtype=torch.float32, device=dev).to(w.torch_dtype())
    kn = torch.randn(shp_k, generator=g, dtype=torch.float32, device=dev).to(w.torch_dtype())
    vn = torch.randn(shp_k, generator=g, dtype=torch.float32, device=dev).to(w.torch_dtype())
    pos_new = (w.context + np.arange(steps, dtype=np.int32))[:, None].repeat(w.batch, axis=1)
    return q, kn, vn, np.ascontiguousarray(pos_new)


# --------------------------------------------------------------------------
# conversions used by callers of the oracle (storage only)
# --------------------------------------------------------------------------
def to_numpy_storage(t: torch.Tensor) -> np.ndarray:
    """fp32 tensor -> fp32 array; bf16 tensor -> uint16 array of its bits."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()
