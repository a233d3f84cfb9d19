"""Seeded synthetic workloads for the FastGen hot path.

This module only *draws inputs*: per-head Q/K/V of a prompt, the decode-time q/k/v stream
and the token classes. It holds none of the method's arithmetic (no softmax, no policy,
no selection), so both the CPU oracle's tests and the HIP path can be fed from it without
sharing anything else. The real workloads of the paper (Llama-1 attention on benchmark
prompts, Sec. 5.1) need weights and datasets; these generators stand in for them with the
same shapes and with attention *structure* planted through reserved dimensions of Q and K
(attention sinks on special tokens, punctuation columns, heavy-hitter columns, a local
band, or nothing), which is the structure Sec. 4 reports for real heads.

Everything is a pure function of (workload, unit index, device type): a unit can be
regenerated on its own, which is how full-size runs hand a sample of units to the oracle.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

# pattern ids
LOCAL, SPECIAL, PUNCT, HEAVY, BROAD = 0, 1, 2, 3, 4
PATTERN_NAMES = ("local", "special", "punct", "heavy", "broad")

CLASS_SPECIAL = 1  # bit 0 of a token-class byte
CLASS_PUNCT = 2    # bit 1

VOCAB = 32000
N_PUNCT_IDS = 16
P_PUNCT = 0.10
ZIPF_A = 1.1


@dataclasses.dataclass(frozen=True)
class Workload:
    """One benchmark configuration. Units are flattened ((b*layers + l)*heads + h)."""
    name: str
    layers: int
    heads: int
    batch: int
    head_dim: int
    dtype: str            # "f32" | "bf16"
    prompt_len: int
    steps: int
    T: float
    r_l: float
    r_f: float
    seed: int
    mix: Tuple[float, float, float, float, float]  # P(local, special, punct, heavy, broad)
    tiny: bool = False    # Tiny config: heads 0..3 carry fixed patterns

    @property
    def num_units(self) -> int:
        return self.batch * self.layers * self.heads

    @property
    def units_per_seq(self) -> int:
        return self.layers * self.heads

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def scaled(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


_UNIFORM = (0.2, 0.2, 0.2, 0.2, 0.2)

WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", 1, 4, 1, 64, "f32", 128, 32, 0.95, 0.1, 0.1, 0, _UNIFORM, tiny=True),
    "llama7b_b1": Workload("llama7b_b1", 32, 32, 1, 128, "bf16", 2048, 256, 0.95, 0.3, 0.3, 1, _UNIFORM),
    "llama7b_b16": Workload("llama7b_b16", 32, 32, 16, 128, "bf16", 1024, 512, 0.95, 0.3, 0.3, 2, _UNIFORM),
    # 60 % local/special-dominated, 40 % broad
    "llama13b_b4": Workload("llama13b_b4", 40, 40, 4, 128, "bf16", 4096, 512, 0.95, 0.3, 0.3, 3,
                            (0.30, 0.30, 0.0, 0.0, 0.40)),
    # 20 % broad (full cache), 50 % special/punct, 30 % local/heavy
    "llama65b_b2": Workload("llama65b_b2", 80, 64, 2, 128, "bf16", 8192, 1024, 0.95, 0.3, 0.3, 4,
                            (0.15, 0.25, 0.25, 0.15, 0.20)),
}


# --------------------------------------------------------------------------------------
# token ids / classes (host side, numpy; tiny amount of data)
# --------------------------------------------------------------------------------------

def punct_id_set(w: Workload) -> np.ndarray:
    rng = np.random.default_rng([w.seed, 11])
    return np.sort(rng.choice(np.arange(1, VOCAB), size=N_PUNCT_IDS, replace=False)).astype(np.int32)


def _draw_ids(rng: np.random.Generator, count: int, punct_ids: np.ndarray) -> np.ndarray:
    """Token ids: with prob. P_PUNCT one of the punctuation ids, else Zipf(1.1) over the rest."""
    others = np.setdiff1d(np.arange(1, VOCAB, dtype=np.int32), punct_ids)
    ranks = np.arange(1, others.size + 1, dtype=np.float64)
    pz = ranks ** (-ZIPF_A)
    pz /= pz.sum()
    ids = others[rng.choice(others.size, size=count, p=pz)]
    is_p = rng.random(count) < P_PUNCT
    ids[is_p] = punct_ids[rng.integers(0, punct_ids.size, size=int(is_p.sum()))]
    return ids.astype(np.int32)


def token_ids(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """(prompt_ids [B,n], decode_ids [S,B]). Id 0 is the one special token (position 0)."""
    pids = punct_id_set(w)
    rng = np.random.default_rng([w.seed, 12])
    prompt = _draw_ids(rng, w.batch * w.prompt_len, pids).reshape(w.batch, w.prompt_len)
    prompt[:, 0] = 0
    dec = _draw_ids(rng, w.steps * w.batch, pids).reshape(w.steps, w.batch)
    return prompt, dec


def classify(ids: np.ndarray, special_ids: Sequence[int], punct_ids: np.ndarray) -> np.ndarray:
    """Token-class bytes (bit 0 special, bit 1 punctuation) from token ids."""
    cls = np.zeros(ids.shape, dtype=np.uint8)
    cls[np.isin(ids, np.asarray(special_ids))] |= CLASS_SPECIAL
    cls[np.isin(ids, punct_ids)] |= CLASS_PUNCT
    return cls


def token_classes(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """(prompt classes [B,n] u8, decode classes [S,B] u8)."""
    p, d = token_ids(w)
    pids = punct_id_set(w)
    return classify(p, [0], pids), classify(d, [0], pids)


# --------------------------------------------------------------------------------------
# per-unit planted structure
# --------------------------------------------------------------------------------------

@dataclasses.dataclass
class UnitPlan:
    pattern: np.ndarray      # [U] int8
    strength: np.ndarray     # [U] float64 (gamma: log-odds-like strength; peak bias for LOCAL)
    heavy_pos: List[Optional[np.ndarray]]  # per unit: sorted heavy-hitter positions or None


def unit_plan(w: Workload) -> UnitPlan:
    U, n = w.num_units, w.prompt_len
    rng = np.random.default_rng([w.seed, 13])
    if w.tiny:
        pattern = np.array([LOCAL, PUNCT, HEAVY, BROAD], dtype=np.int8)[np.arange(U) % 4]
        strength = np.array([8.0, 6.0, 4.0, 0.0])[np.arange(U) % 4]
    else:
        pattern = rng.choice(5, size=U, p=np.asarray(w.mix) / np.sum(w.mix)).astype(np.int8)
        strength = rng.uniform(1.5, 4.5, size=U)
        strength[pattern == LOCAL] = rng.uniform(6.0, 10.0, size=int((pattern == LOCAL).sum()))
    heavy: List[Optional[np.ndarray]] = [None] * U
    n_heavy = min(n - 1, 8 if w.tiny else max(8, n // 16))
    for u in np.nonzero(pattern == HEAVY)[0]:
        r = np.random.default_rng([w.seed, 14, int(u)])
        heavy[u] = np.sort(r.choice(np.arange(1, n), size=n_heavy, replace=False)).astype(np.int64)
    return UnitPlan(pattern, strength, heavy)


def _column_beta(w: Workload, pattern: int, gamma: float) -> float:
    """Additive logit bias on the favoured columns. For the non-tiny workloads `gamma`
    is the log-odds of favoured-vs-other mass for a late query row, so the same gamma
    range straddles the recovery threshold at every prompt length."""
    if w.tiny:
        return gamma
    n = w.prompt_len
    if pattern == SPECIAL:
        return math.log(n) + gamma
    if pattern == PUNCT:
        return math.log((1.0 - P_PUNCT) / P_PUNCT) + gamma
    return math.log(15.0) + gamma  # HEAVY: 1/16 of the columns


def _local_series(w: Workload, peak: float, device) -> Tuple[torch.Tensor, torch.Tensor, int]:
    """Amplitudes a_m and angular steps for the band bias  sum_m a_m^2 cos(pi m (i-j)/N)."""
    n, S, d = w.prompt_len, w.steps, w.head_dim
    N = n + S
    window = 16.0 if w.tiny else 0.6 * max(1.0, math.floor(w.r_l * n))
    sigma = window / 2.5
    m_sigma = N / (math.pi * sigma)
    M = int(min(math.ceil(2.5 * m_sigma), d // 4))
    m = torch.arange(1, M + 1, dtype=torch.float64)
    g = torch.exp(-(m * m) / (2.0 * m_sigma * m_sigma))
    a2 = peak * math.sqrt(d) * g / g.sum()
    return torch.sqrt(a2).to(device), (math.pi * m / N).to(device), M


def _gen(device, *key: int) -> torch.Generator:
    g = torch.Generator(device=device)
    seed = 0
    for k in key:
        seed = (seed * 1_000_003 + int(k) + 0x9E3779B97F4A7C15) % (2 ** 63 - 1)
    g.manual_seed(seed)
    return g


def _plant(w: Workload, plan: UnitPlan, u: int, Q: torch.Tensor, K: torch.Tensor,
           pos: torch.Tensor, cls_row: torch.Tensor) -> None:
    """Overwrite the reserved dimensions of Q and K (rows at absolute positions `pos`,
    token classes `cls_row`) so that scale*q.k gains the unit's planted bias."""
    pat = int(plan.pattern[u])
    d = w.head_dim
    if pat == BROAD:
        return
    if pat == LOCAL:
        a, om, M = _local_series(w, float(plan.strength[u]), Q.device)
        ang = pos.to(torch.float64)[:, None] * om[None, :]
        c, s = (a * torch.cos(ang)).to(Q.dtype), (a * torch.sin(ang)).to(Q.dtype)
        Q[:, 0:2 * M:2], Q[:, 1:2 * M:2] = c, s
        K[:, 0:2 * M:2], K[:, 1:2 * M:2] = c, s
        return
    beta = _column_beta(w, pat, float(plan.strength[u]))
    alpha = math.sqrt(beta * math.sqrt(d))
    if pat == SPECIAL:
        fav = (cls_row & CLASS_SPECIAL) != 0
    elif pat == PUNCT:
        fav = (cls_row & (CLASS_SPECIAL | CLASS_PUNCT)) != 0
    else:
        hp = torch.as_tensor(plan.heavy_pos[u], device=Q.device)
        fav = torch.isin(pos, hp)
    Q[:, 0] = alpha
    K[:, 0] = torch.where(fav, alpha, 0.0).to(K.dtype)


def prompt_unit(w: Workload, plan: UnitPlan, cls_prompt: np.ndarray, u: int, device="cpu"
                ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Q, K, V [n, d] of unit u in the workload's dtype."""
    n, d = w.prompt_len, w.head_dim
    g = _gen(device, w.seed, 21, u)
    x = torch.randn((3, n, d), generator=g, device=device, dtype=torch.float32)
    Q, K, V = x[0], x[1], x[2]
    b = u // w.units_per_seq
    pos = torch.arange(n, device=device)
    _plant(w, plan, u, Q, K, pos, torch.as_tensor(cls_prompt[b], device=device))
    dt = w.torch_dtype
    return Q.to(dt), K.to(dt), V.to(dt)


def decode_unit(w: Workload, plan: UnitPlan, cls_decode: np.ndarray, u: int, device="cpu"
                ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """q, k, v [S, d] of unit u for decode steps t = 0..S-1 (absolute positions n+t)."""
    n, S, d = w.prompt_len, w.steps, w.head_dim
    g = _gen(device, w.seed, 22, u)
    x = torch.randn((3, S, d), generator=g, device=device, dtype=torch.float32)
    q, k, v = x[0], x[1], x[2]
    b = u // w.units_per_seq
    pos = torch.arange(n, n + S, device=device)
    _plant(w, plan, u, q, k, pos, torch.as_tensor(cls_decode[:, b], device=device))
    dt = w.torch_dtype
    return q.to(dt), k.to(dt), v.to(dt)


def prompt_group_queries(w: Workload, plan: UnitPlan, cls_prompt: np.ndarray, u: int, G: int,
                         device="cpu") -> torch.Tensor:
    """Q [G, n, d]: the query heads that share K/V head u. Head 0 is prompt_unit's Q; the
    others draw fresh noise and carry the same planted dimensions (same attention pattern)."""
    n, d = w.prompt_len, w.head_dim
    out = torch.empty((G, n, d), dtype=w.torch_dtype, device=device)
    out[0] = prompt_unit(w, plan, cls_prompt, u, device)[0]
    b = u // w.units_per_seq
    pos = torch.arange(n, device=device)
    for h in range(1, G):
        Q = torch.randn((n, d), generator=_gen(device, w.seed, 23, u, h), device=device, dtype=torch.float32)
        _plant(w, plan, u, Q, torch.empty_like(Q), pos, torch.as_tensor(cls_prompt[b], device=device))
        out[h] = Q.to(w.torch_dtype)
    return out


def decode_group_queries(w: Workload, plan: UnitPlan, cls_decode: np.ndarray, u: int, G: int,
                         device="cpu") -> torch.Tensor:
    """q [S, G, d] for the decode steps, head 0 = decode_unit's q."""
    n, S, d = w.prompt_len, w.steps, w.head_dim
    out = torch.empty((S, G, d), dtype=w.torch_dtype, device=device)
    out[:, 0] = decode_unit(w, plan, cls_decode, u, device)[0]
    b = u // w.units_per_seq
    pos = torch.arange(n, n + S, device=device)
    for h in range(1, G):
        q = torch.randn((S, d), generator=_gen(device, w.seed, 24, u, h), device=device, dtype=torch.float32)
        _plant(w, plan, u, q, torch.empty_like(q), pos, torch.as_tensor(cls_decode[:, b], device=device))
        out[:, h] = q.to(w.torch_dtype)
    return out


def prompt_batch(w: Workload, plan: UnitPlan, cls_prompt: np.ndarray, units: Sequence[int],
                 device="cpu") -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Q, K, V [len(units), n, d] for the given units."""
    m, n, d = len(units), w.prompt_len, w.head_dim
    Q = torch.empty((m, n, d), dtype=w.torch_dtype, device=device)
    K = torch.empty_like(Q)
    V = torch.empty_like(Q)
    for i, u in enumerate(units):
        Q[i], K[i], V[i] = prompt_unit(w, plan, cls_prompt, int(u), device)
    return Q, K, V


def decode_batch(w: Workload, plan: UnitPlan, cls_decode: np.ndarray, units: Sequence[int],
                 device="cpu") -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """q, k, v [S, len(units), d] (step-major, as the decode call consumes them)."""
    m, S, d = len(units), w.steps, w.head_dim
    q = torch.empty((S, m, d), dtype=w.torch_dtype, device=device)
    k = torch.empty_like(q)
    v = torch.empty_like(q)
    for i, u in enumerate(units):
        q[:, i], k[:, i], v[:, i] = decode_unit(w, plan, cls_decode, int(u), device)
    return q, k, v


def to_f64(x: torch.Tensor) -> np.ndarray:
    """Exact widening of a (bf16 or f32) tensor to a float64 numpy array on the host."""
    return x.detach().to("cpu").to(torch.float64).numpy()
