"""FastGen hot path -- plain float64 CPU oracle.  TEST INFRASTRUCTURE ONLY.

This file is the checker, not the product. Only tests, the smoke check and the benchmark's
CPU-baseline leg may import it; the HIP library never does, and nothing here imports the HIP
library or shares code, tables or constants with it.

It writes out, densely and in float64, what the paper defines for ONE attention head
("unit") at a time:

  * Alg. 1 / Sec. 3.3: the attention map A = softmax(Q K^T) of the prompt (causal,
    scaled -- decoder-only attention, Sec. 3.1);
  * Sec. 3.4: the four base policies (special, punctuation, local, frequent) and the
    hybrid policy family of Eq. 2, "+" meaning union of kept sets;
  * Eq. 1: the cheapest policy of the family whose recovery reaches T;
  * Alg. 1: the compressed cache f(K, V, C);
  * Alg. 2: one decode step over the compressed cache followed by re-application of f.

Readings taken where the paper is silent (each is a *reading*, stated once here):
  R1  softmax is causal and uses a scale (default 1/sqrt(d)).
  R2  the norm in Eq. 1 is the mean over query rows of the total-variation distance between
      a row of A and the same row restricted to the kept tokens and renormalised; that
      distance equals 1 - (kept mass of the row), so "recovers A with ratio T" <=> the mean
      kept attention mass is >= T (matches Sec. 4: "accumulated attention score on special
      tokens is higher than 0.95").
  R3  on the prompt, `frequent` is the hindsight top-k of the complete column sums and
      `local` is row-relative (row i keeps columns i-w+1..i).
  R4  frequent's budget is counted over all held tokens and then united with the other sets
      (overlap allowed); k_f(L) = floor(r_f * L) follows the *current* length L, the local
      window w = max(1, floor(r_l * n)) is fixed by the *input* length n (Sec. 3.4).
  R5  budgets are floor() of the IEEE-double product.
  R6  ties: equal cost -> smaller policy id; equal score -> keep the smaller position.
  R7  decode step t handles a new token at position n+t; it attends to itself; its score
      starts at 0 and receives this step's attention like every other held token; scores
      are only maintained for policies that contain `frequent`.
  R8  R >= T (non-strict), as Eq. 1's "<=".
  R13 grouped-query attention (named future work in Sec. 5.1 and the Conclusion, no rule
      given): G query heads share one K/V head and therefore one cache and one policy. The
      extension taken here reduces to the paper at G = 1: Eq. 1 averages over the rows of
      all G heads (recovery = mean kept mass over the G*n rows), a token's cumulative
      attention score is the sum over the G heads, every head attends over the shared
      compressed cache while decoding, and a step adds the G attention rows to the scores.

Pinned by tests/test_oracle_pins.py (closed forms for Q = 0, brute force over subsets,
textbook softmax/attention, TV-distance identity, nestedness, full-cache invariants).
Parity unpinned (no number in the paper distinguishes the alternatives): readings R3, R4,
R6, R7 themselves.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

POLICY_NAMES = ("special", "special+punct", "special+punct+frequent",
                "special+punct+frequent+local", "full")
N_POLICIES = 5
CLASS_SPECIAL = 1
CLASS_PUNCT = 2

# A policy family is four component masks plus C_full (policy id 4). Components (Sec. 3.4):
# bit 0 special, bit 1 punctuation, bit 2 frequent, bit 3 local; mask 0 = slot not used.
# The default is the family of Eq. 2; App. A.1 (Tables 4 and 5) varies the members and the
# order in which components are added, and Sec. 5.1 uses single members as fixed baselines.
SPECIAL, PUNCT, FREQUENT, LOCAL = 1, 2, 4, 8
DEFAULT_FAMILY = (SPECIAL, SPECIAL | PUNCT, SPECIAL | PUNCT | FREQUENT, SPECIAL | PUNCT | FREQUENT | LOCAL)


# ----------------------------------------------------------------------------------------
# budgets (Sec. 3.4: ratios r_l, r_f)
# ----------------------------------------------------------------------------------------

def local_window(r_l: float, n: int) -> int:
    """w: length budget of local context, a ratio of the INPUT sequence length."""
    return max(1, int(math.floor(float(r_l) * float(n))))


def frequent_budget(r_f: float, L: int) -> int:
    """k_f(L): length budget of frequent tokens, a ratio of the CURRENT sequence length."""
    return int(math.floor(float(r_f) * float(L)))


# ----------------------------------------------------------------------------------------
# Sec. 3.4: which tokens C_special and C_punct. keep
# ----------------------------------------------------------------------------------------

def classify_tokens(token_ids, special_ids, punct_ids) -> np.ndarray:
    """Class byte of every token: bit 0 if the token is a special token (e.g. the
    begin-of-sentence or instruction markers), bit 1 if it is a punctuation token."""
    ids = np.asarray(token_ids)
    special, punct = set(int(x) for x in special_ids), set(int(x) for x in punct_ids)
    out = np.zeros(ids.shape, dtype=np.uint8)
    for idx in np.ndindex(ids.shape):
        t = int(ids[idx])
        out[idx] = (CLASS_SPECIAL if t in special else 0) | (CLASS_PUNCT if t in punct else 0)
    return out


# ----------------------------------------------------------------------------------------
# Alg. 1, line "A <- softmax(Q K^T)"
# ----------------------------------------------------------------------------------------

def attention_map(Q: np.ndarray, K: np.ndarray, scale: float) -> np.ndarray:
    """Dense causal attention map of one head, float64, rows sum to 1."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    n = Q.shape[0]
    s = (Q @ K.T) * float(scale)
    causal = np.tril(np.ones((n, n), dtype=bool))
    s = np.where(causal, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=1, keepdims=True)


def top_k_positions(score: np.ndarray, pos: np.ndarray, k: int) -> np.ndarray:
    """Positions of the k largest scores; equal scores -> the smaller position wins."""
    if k <= 0:
        return np.zeros(0, dtype=np.int64)
    order = np.lexsort((pos, -score))       # primary -score, secondary pos
    return np.sort(pos[order[:k]])


def boundary_gap(score: np.ndarray, k: int) -> float:
    """Relative gap between the k-th and (k+1)-th largest score (inf if no boundary)."""
    m = score.size
    if k <= 0 or k >= m:
        return math.inf
    s = np.sort(score)[::-1]
    hi, lo = s[k - 1], s[k]
    return float((hi - lo) / hi) if hi > 0 else 0.0


# ----------------------------------------------------------------------------------------
# Sec. 3.4 policies on the prompt, Eq. 2 family, Eq. 1 selection
# ----------------------------------------------------------------------------------------

@dataclass
class Profile:
    policy: int
    recovery: np.ndarray        # [5] float64, R_c
    cost: np.ndarray            # [5] int64, |K_c| at the end of the prompt
    kept: np.ndarray            # sorted positions of K_policy
    colsum: np.ndarray          # [n] cumulative attention score of every prompt token
    window: int
    k_f: int
    margin: float               # min_c<4 |R_c - T|
    topk_gap: float             # relative gap at the frequent boundary
    sets: List[np.ndarray] = field(default_factory=list)  # K_0..K_4 (sorted positions)


def component_sets(cls: np.ndarray, colsum: np.ndarray, r_l: float, r_f: float) -> Dict[int, np.ndarray]:
    """The four base kept sets at the end of the prompt (Sec. 3.4)."""
    n = colsum.size
    pos = np.arange(n, dtype=np.int64)
    w = local_window(r_l, n)
    return {SPECIAL: pos[(cls & CLASS_SPECIAL) != 0],
            PUNCT: pos[(cls & CLASS_PUNCT) != 0],
            FREQUENT: top_k_positions(colsum, pos, frequent_budget(r_f, n)),
            LOCAL: pos[max(0, n - w):]}


def kept_sets(cls: np.ndarray, colsum: np.ndarray, r_l: float, r_f: float,
              family=DEFAULT_FAMILY) -> List[np.ndarray]:
    """K_0..K_4 at the end of the prompt: "+" is the union of the components' kept sets."""
    n = colsum.size
    comp = component_sets(cls, colsum, r_l, r_f)
    out = []
    for mask in family:
        k = np.zeros(0, dtype=np.int64)
        for bit in (SPECIAL, PUNCT, FREQUENT, LOCAL):
            if mask & bit:
                k = np.union1d(k, comp[bit])
        out.append(k)
    out.append(np.arange(n, dtype=np.int64))
    return out


def recovery_dense(A: np.ndarray, static_keep: np.ndarray, window: int) -> float:
    """Mean over query rows of the attention mass on kept tokens. `static_keep` is a
    boolean column mask; window > 0 additionally keeps columns i-window+1..i of row i."""
    n = A.shape[0]
    i = np.arange(n)[:, None]
    j = np.arange(n)[None, :]
    keep = np.broadcast_to(static_keep[None, :], (n, n)) & (j <= i)
    if window > 0:
        keep = keep | ((j <= i) & (j > i - window))
    kept_mass_per_row = np.where(keep, A, 0.0).sum(axis=1)
    return float(kept_mass_per_row.mean())


def select_policy(cost: np.ndarray, recovery: np.ndarray, T: float, usable=None) -> int:
    """Eq. 1: argmin cost subject to recovery >= T; equal cost -> smaller id."""
    best = -1
    for c in range(N_POLICIES):
        if usable is not None and not usable[c]:
            continue
        # C_full is the uncompressed cache: its difference to A is zero by definition
        feasible = (c == N_POLICIES - 1) or (recovery[c] >= T)
        if feasible and (best < 0 or cost[c] < cost[best]):
            best = c
    return best


def profile_unit(Q: np.ndarray, K: np.ndarray, cls: np.ndarray, T: float, r_l: float,
                 r_f: float, scale: float, forced_policy: int = -1, family=DEFAULT_FAMILY) -> Profile:
    """Alg. 1 up to the choice of C for one K/V head. Q is [n, d], or [G, n, d] for the G
    query heads that share it (R13)."""
    Qg = np.asarray(Q, dtype=np.float64)
    Qg = Qg[None] if Qg.ndim == 2 else Qg          # [G, n, d]: the query heads sharing this K/V head
    maps = [attention_map(Qh, K, scale) for Qh in Qg]
    n = maps[0].shape[0]
    colsum = np.sum([A.sum(axis=0) for A in maps], axis=0)
    cls = np.asarray(cls)
    sets = kept_sets(cls, colsum, r_l, r_f, family)
    comp = component_sets(cls, colsum, r_l, r_f)
    w = local_window(r_l, n)
    rec = np.zeros(N_POLICIES)
    usable = [m != 0 for m in family] + [True]
    for c in range(N_POLICIES):
        static = np.zeros(n, dtype=bool)
        if c == 4:
            static[:] = True
        else:
            # the local component is row-relative on the prompt; the others are static column sets
            for bit in (SPECIAL, PUNCT, FREQUENT):
                if family[c] & bit:
                    static[comp[bit]] = True
        window = w if (c < 4 and family[c] & LOCAL) else 0
        rec[c] = float(np.mean([recovery_dense(A, static, window) for A in maps]))
    cost = np.array([s.size for s in sets], dtype=np.int64)
    policy = select_policy(cost, rec, T, usable) if forced_policy < 0 else int(forced_policy)
    margins = [abs(rec[c] - T) for c in range(4) if usable[c]]
    return Profile(policy=policy, recovery=rec, cost=cost, kept=sets[policy], colsum=colsum,
                   window=w, k_f=frequent_budget(r_f, n),
                   margin=float(min(margins)) if margins else math.inf,
                   topk_gap=boundary_gap(colsum, frequent_budget(r_f, n)), sets=sets)


# ----------------------------------------------------------------------------------------
# Alg. 1 compaction f(K, V, C) and Alg. 2 decode step
# ----------------------------------------------------------------------------------------

@dataclass
class Cache:
    """Compressed cache of one head: held tokens in ascending position order."""
    policy: int
    n: int                      # prompt length (fixes the local window)
    K: np.ndarray               # [len, d]
    V: np.ndarray               # [len, d]
    score: np.ndarray           # [len] cumulative attention score
    pos: np.ndarray             # [len] int64
    cls: np.ndarray             # [len] uint8
    mask: int = 0               # component mask of the policy (ignored for C_full)
    min_gap: float = math.inf   # smallest relative top-k boundary gap seen while decoding
    probe: Optional[np.ndarray] = None  # step_recovery() of the last probed step
    probe_gap: float = math.inf         # relative top-k boundary gap of that step
    fragile_step: int = -1      # first decode step whose boundary gap fell below `gap_eps`


def compact_unit(K: np.ndarray, V: np.ndarray, cls: np.ndarray, prof: Profile,
                 family=DEFAULT_FAMILY) -> Cache:
    keep = prof.kept
    return Cache(policy=prof.policy, n=K.shape[0], mask=family[prof.policy] if prof.policy < 4 else 0,
                 K=np.asarray(K, dtype=np.float64)[keep].copy(),
                 V=np.asarray(V, dtype=np.float64)[keep].copy(),
                 score=prof.colsum[keep].copy(), pos=keep.copy(),
                 cls=np.asarray(cls, dtype=np.uint8)[keep].copy())


def kept_after_step(policy: int, mask: int, pos: np.ndarray, cls: np.ndarray, score: np.ndarray,
                    p_new: int, window: int, r_f: float) -> np.ndarray:
    """Boolean mask over held tokens: which stay after the token at position p_new."""
    if policy == 4:
        return np.ones(pos.size, dtype=bool)
    keep = np.zeros(pos.size, dtype=bool)
    if mask & SPECIAL:
        keep |= (cls & CLASS_SPECIAL) != 0
    if mask & PUNCT:
        keep |= (cls & CLASS_PUNCT) != 0
    if mask & FREQUENT:
        top = top_k_positions(score, pos, frequent_budget(r_f, p_new + 1))
        keep |= np.isin(pos, top)
    if mask & LOCAL:
        keep |= pos > p_new - window
    return keep


def step_recovery(c: Cache, a: np.ndarray, p: int, r_l: float, r_f: float, family) -> np.ndarray:
    """Stability probe (Sec. 4, accumulated attention score at later decoding steps): the mass
    the new token's attention row `a` (the mean of the G rows for grouped heads) puts on each family member's tokens among the tokens held
    during the step. Members as in Sec. 3.4 at length p + 1: special / punctuation by class,
    frequent = top k_f(p + 1) cumulative scores (this step's attention included), local =
    the last w positions. Entry 4 (C_full) is the whole row."""
    w = local_window(r_l, c.n)
    top = top_k_positions(c.score, c.pos, frequent_budget(r_f, p + 1))
    member = {SPECIAL: (c.cls & CLASS_SPECIAL) != 0, PUNCT: (c.cls & CLASS_PUNCT) != 0,
              FREQUENT: np.isin(c.pos, top), LOCAL: c.pos > p - w}
    rho = np.zeros(N_POLICIES)
    for i, mask in enumerate(family):
        inside = np.zeros(c.pos.size, dtype=bool)
        for bit in (SPECIAL, PUNCT, FREQUENT, LOCAL):
            if mask & bit:
                inside |= member[bit]
        rho[i] = a[inside].sum()
    rho[4] = a.sum()
    return rho


def decode_step(c: Cache, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, cls_new: int,
                t: int, r_l: float, r_f: float, scale: float, gap_eps: float = 0.0,
                probe_family=None) -> np.ndarray:
    """One pass of Alg. 2's inner body for one K/V head; q is [d], or [G, d] for the query
    heads sharing it; returns the attention output o ([d] or [G, d]). With
    `probe_family` the cumulative scores are kept for every policy and c.probe receives
    step_recovery() of this step."""
    p = c.n + t
    c.K = np.vstack([c.K, np.asarray(k_new, dtype=np.float64)[None, :]])
    c.V = np.vstack([c.V, np.asarray(v_new, dtype=np.float64)[None, :]])
    c.score = np.append(c.score, 0.0)
    c.pos = np.append(c.pos, p)
    c.cls = np.append(c.cls, np.uint8(cls_new))
    qg = np.asarray(q, dtype=np.float64)
    single = qg.ndim == 1
    qg = qg[None] if single else qg                # [G, d]
    s = (qg @ c.K.T) * float(scale)                # [G, len]
    e = np.exp(s - s.max(axis=1, keepdims=True))
    ag = e / e.sum(axis=1, keepdims=True)          # one attention row per query head
    o = ag @ c.V
    o = o[0] if single else o
    a = ag.sum(axis=0)                             # what the step adds to the cumulative scores
    uses_scores = c.policy < 4 and (c.mask & FREQUENT) != 0
    if uses_scores or probe_family is not None:
        c.score = c.score + a   # Sec. 3.4: cumulative attention score of every held token
    if probe_family is not None:
        c.probe = step_recovery(c, a / ag.shape[0], p, r_l, r_f, probe_family)
        c.probe_gap = boundary_gap(c.score, frequent_budget(r_f, p + 1))
    if uses_scores:
        g = boundary_gap(c.score, frequent_budget(r_f, p + 1))
        c.min_gap = min(c.min_gap, g)
        if g < gap_eps and c.fragile_step < 0:
            c.fragile_step = t
    keep = kept_after_step(c.policy, c.mask, c.pos, c.cls, c.score, p, local_window(r_l, c.n), r_f)
    c.K, c.V, c.score, c.pos, c.cls = c.K[keep], c.V[keep], c.score[keep], c.pos[keep], c.cls[keep]
    return o


def run_unit(Q, K, V, cls, q_steps, k_steps, v_steps, cls_steps, T, r_l, r_f, scale,
             forced_policy: int = -1, gap_eps: float = 0.0, record_states: bool = False,
             family=DEFAULT_FAMILY, probe=False) -> Dict:
    """Whole path for one head: profile, compact, S decode steps. `probe`: True (every step)
    or the set of decode steps that run with the stability probe."""
    prof = profile_unit(Q, K, cls, T, r_l, r_f, scale, forced_policy, family)
    cache = compact_unit(K, V, cls, prof, family)
    S = 0 if q_steps is None else len(q_steps)
    d = np.asarray(K).shape[1]
    outs = np.zeros((S, d)) if S == 0 or np.asarray(q_steps[0]).ndim == 1 else np.zeros((S, len(q_steps[0]), d))
    lens = np.zeros(S, dtype=np.int64)
    states: List[np.ndarray] = []
    score_states: List[np.ndarray] = []
    init_pos = cache.pos.copy()
    probed = (lambda t: bool(probe)) if isinstance(probe, bool) else (lambda t: t in probe)
    probes = np.zeros((S, N_POLICIES))
    probe_gaps = np.full(S, math.inf)
    for t in range(S):
        outs[t] = decode_step(cache, q_steps[t], k_steps[t], v_steps[t], int(cls_steps[t]),
                              t, r_l, r_f, scale, gap_eps, family if probed(t) else None)
        if probed(t):
            probes[t], probe_gaps[t] = cache.probe, cache.probe_gap
        lens[t] = cache.pos.size
        if record_states:
            states.append(cache.pos.copy())
            score_states.append(cache.score.copy())
    return dict(profile=prof, init_pos=init_pos, outs=outs, lens=lens, states=states,
                score_states=score_states, cache=cache, probes=probes, probe_gaps=probe_gaps)
