"""Pins for the float64 oracle: every check here compares the oracle with something that
is NOT the oracle -- exact rational closed forms, brute force over subsets, textbook
softmax/attention from another library, or a from-scratch recomputation by loops."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import fastgen_oracle as fo

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_unit(seed, n, d, p_punct=0.15, bias=None):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((n, d))
    K = rng.standard_normal((n, d))
    V = rng.standard_normal((n, d))
    cls = np.zeros(n, dtype=np.uint8)
    cls[0] = 1
    cls[1:][rng.random(n - 1) < p_punct] = 2
    if bias is not None:
        K[:, 0] = np.where(cls != 0, bias, 0.0)
        Q[:, 0] = 1.0
    return Q, K, V, cls


def harmonic(k):
    return sum(Fraction(1, i) for i in range(1, k + 1))


# ---------------------------------------------------------------- A (Alg. 1, Sec. 3.3)

def test_attention_map_is_textbook_causal_softmax():
    Q, K, _, _ = rand_unit(1, 37, 16)
    scale = 0.25
    A = fo.attention_map(Q, K, scale)
    s = torch.from_numpy(Q) @ torch.from_numpy(K).T * scale
    s = s.masked_fill(torch.triu(torch.ones(37, 37, dtype=torch.bool), 1), float("-inf"))
    ref = torch.softmax(s, dim=1).numpy()
    assert np.allclose(A, ref, rtol=0, atol=1e-14)
    assert np.allclose(A.sum(1), 1.0, atol=1e-14)
    assert np.all(A[np.triu_indices(37, 1)] == 0.0)
    assert abs(A.sum() - 37) < 1e-12          # sum_j colsum_j = n
    # Q K^T, not K Q^T: row i is the distribution of QUERY i
    i = 20
    row = np.exp(scale * (K[: i + 1] @ Q[i]))
    assert np.allclose(A[i, : i + 1], row / row.sum(), atol=1e-14)


def test_golden_q0_n4_worked_example():
    """Uniform causal attention (Q = 0): A_ij = 1/(i+1). Values derived by hand in exact
    rationals and stored in tests/golden/q0_n4.txt."""
    vals = {}
    with open(os.path.join(GOLDEN, "q0_n4.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split("=")
            vals[k.strip()] = [Fraction(x) for x in v.split()]
    n, d = 4, 8
    Q = np.zeros((n, d))
    K = np.random.default_rng(0).standard_normal((n, d))
    cls = np.array([1, 0, 0, 0], dtype=np.uint8)
    A = fo.attention_map(Q, K, 1.0)
    assert np.allclose(A.sum(0), [float(x) for x in vals["colsum"]], atol=1e-15)
    keep0 = np.array([True, False, False, False])
    assert abs(fo.recovery_dense(A, keep0, 0) - float(vals["R_special"][0])) < 1e-15
    assert abs(fo.recovery_dense(A, keep0, 1) - float(vals["R_special_local_w1"][0])) < 1e-15
    # frequent with k_f = 2 -> positions {0, 1}
    assert list(fo.top_k_positions(A.sum(0), np.arange(4), 2)) == [0, 1]
    keepf = np.array([True, True, False, False])
    assert abs(fo.recovery_dense(A, keepf, 0) - float(vals["R_freq_k2"][0])) < 1e-15
    # through the full profile: r_f = 0.5 -> k_f = 2, r_l = 0.25 -> w = 1
    p = fo.profile_unit(Q, K, cls, 0.75, 0.25, 0.5, 1.0)
    assert p.k_f == 2 and p.window == 1
    assert np.allclose(p.recovery, [float(x) for x in vals["R_family"]], atol=1e-15)
    assert list(p.cost) == [1, 1, 2, 3, 4]
    assert p.policy == 2            # 38/48 >= 0.75, cost 2
    assert list(p.kept) == [0, 1]


@pytest.mark.parametrize("n,w,k", [(9, 3, 2), (64, 7, 19), (50, 50, 0)])
def test_q0_closed_forms_harmonic(n, w, k):
    """Q = 0: colsum_j = H_n - H_j, band sum_j = H_min(j+w,n) - H_j; frequent = first k."""
    Q = np.zeros((n, 4))
    K = np.ones((n, 4))
    A = fo.attention_map(Q, K, 0.5)
    H = [harmonic(i) for i in range(n + 1)]
    colsum = [H[n] - H[j] for j in range(n)]
    assert np.allclose(A.sum(0), [float(c) for c in colsum], atol=1e-13)
    top = fo.top_k_positions(A.sum(0), np.arange(n), k)
    assert list(top) == list(range(k))
    static = np.zeros(n, dtype=bool)
    static[:k] = True
    band = [H[min(j + w, n)] - H[j] for j in range(n)]
    expect = (sum(colsum[:k]) + sum(band[k:])) / n
    assert abs(fo.recovery_dense(A, static, w) - float(expect)) < 1e-13
    expect_static = sum(colsum[:k]) / n
    assert abs(fo.recovery_dense(A, static, 0) - float(expect_static)) < 1e-13


def test_one_hot_head_selects_special():
    Q, K, _, cls = rand_unit(3, 40, 8, bias=None)
    K[:, 0] = 0.0
    K[0, 0] = 200.0
    Q[:, 0] = 1.0
    p = fo.profile_unit(Q, K, cls, 0.95, 0.3, 0.3, 1.0)
    assert p.policy == 0 and abs(p.recovery[0] - 1.0) < 1e-12
    assert list(p.kept) == [0]


# ---------------------------------------------------------------- Eq. 1 <=> kept mass

@pytest.mark.parametrize("seed", [0, 1, 2])
def test_eq1_distance_equals_one_minus_kept_mass(seed):
    """Brute force of Eq. 1's constraint: softmax over the kept keys only, half the L1
    distance to the full row, averaged over rows == 1 - R_c."""
    n, d = 24, 8
    Q, K, _, cls = rand_unit(seed, n, d, bias=2.0)
    scale = 1 / math.sqrt(d)
    prof = fo.profile_unit(Q, K, cls, 0.9, 0.25, 0.25, scale)
    A = fo.attention_map(Q, K, scale)
    w = prof.window
    for c in range(5):
        static = set(prof.sets[min(c, 2)].tolist()) if c < 4 else set(range(n))
        dist = 0.0
        for i in range(n):
            kept = {j for j in static if j <= i}
            if c == 3:
                kept |= {j for j in range(max(0, i - w + 1), i + 1)}
            kept = sorted(kept)
            assert kept, "position 0 is special"
            logits = np.array([scale * Q[i] @ K[j] for j in kept])
            e = np.exp(logits - logits.max())
            a_c = np.zeros(n)
            a_c[kept] = e / e.sum()
            dist += 0.5 * np.abs(A[i] - a_c).sum()
        assert abs(dist / n - (1.0 - prof.recovery[c])) < 1e-12


@pytest.mark.parametrize("seed", range(4))
def test_dense_recovery_equals_column_and_band_sums(seed):
    n, d = 33, 8
    Q, K, _, cls = rand_unit(10 + seed, n, d, bias=1.5)
    prof = fo.profile_unit(Q, K, cls, 0.9, 0.2, 0.3, 0.3)
    A = fo.attention_map(Q, K, 0.3)
    w = prof.window
    colsum = np.array([sum(A[i, j] for i in range(n)) for j in range(n)])
    band = np.array([sum(A[i, j] for i in range(j, min(j + w, n))) for j in range(n)])
    assert np.allclose(prof.colsum, colsum, atol=1e-14)
    for c in range(3):
        assert abs(prof.recovery[c] - colsum[prof.sets[c]].sum() / n) < 1e-13
    in2 = np.zeros(n, dtype=bool)
    in2[prof.sets[2]] = True
    r3 = (colsum[in2].sum() + band[~in2].sum()) / n
    assert abs(prof.recovery[3] - r3) < 1e-13
    assert abs(prof.recovery[4] - 1.0) < 1e-14


@pytest.mark.parametrize("seed", range(6))
def test_nested_sets_and_monotone(seed):
    n, d = 48, 8
    Q, K, _, cls = rand_unit(20 + seed, n, d, bias=float(seed))
    prof = fo.profile_unit(Q, K, cls, 0.95, 0.3, 0.3, 0.35)
    for a, b in zip(prof.sets[:-1], prof.sets[1:]):
        assert set(a.tolist()) <= set(b.tolist())
    assert np.all(np.diff(prof.cost) >= 0)
    assert np.all(np.diff(prof.recovery) >= -1e-15)
    assert prof.cost[4] == n and abs(prof.recovery[4] - 1) < 1e-14
    assert list(prof.kept) == sorted(prof.sets[prof.policy].tolist())


# ---------------------------------------------------------------- selection (Eq. 1 / Eq. 2)

@pytest.mark.parametrize("seed", range(8))
def test_selection_matches_brute_force_over_unions(seed):
    """All 16 unions of {special, punct, frequent, local}: cost and recovery from dense A by
    loops. Restricted to the members of Eq. 2's family the literal argmin equals both the
    oracle's choice and the greedy first-hit scan (App. A.1)."""
    n, d = 20, 4
    T = [0.6, 0.8, 0.9, 0.95][seed % 4]
    Q, K, _, cls = rand_unit(40 + seed, n, d, p_punct=0.2, bias=[0.0, 2.0, 4.0, 8.0][seed // 2])
    scale, r_l, r_f = 0.5, 0.25, 0.2
    prof = fo.profile_unit(Q, K, cls, T, r_l, r_f, scale)
    A = fo.attention_map(Q, K, scale)
    w = max(1, math.floor(r_l * n))
    k = math.floor(r_f * n)
    colsum = A.sum(0)
    ranked = sorted(range(n), key=lambda j: (-colsum[j], j))
    base = {
        "s": {j for j in range(n) if cls[j] & 1},
        "p": {j for j in range(n) if cls[j] & 2},
        "f": set(ranked[:k]),
    }
    table = {}
    for r in range(5):
        for combo in itertools.combinations("spfl", r):
            static = set().union(*[base[x] for x in combo if x != "l"]) if combo else set()
            use_local = "l" in combo
            end_set = static | (set(range(n - w, n)) if use_local else set())
            rec = 0.0
            for i in range(n):
                cols = {j for j in static if j <= i}
                if use_local:
                    cols |= set(range(max(0, i - w + 1), i + 1))
                rec += sum(A[i, j] for j in cols)
            table["".join(combo)] = (len(end_set), rec / n)
    family = ["s", "sp", "spf", "spfl"]
    cands = [(table[f][0], c) for c, f in enumerate(family) if table[f][1] >= T] + [(n, 4)]
    brute = min(cands)[1]
    first_hit = next((c for c, f in enumerate(family) if table[f][1] >= T), 4)
    assert prof.policy == brute == first_hit
    for c, f in enumerate(family):
        assert prof.cost[c] == table[f][0]
        assert abs(prof.recovery[c] - table[f][1]) < 1e-13


@pytest.mark.parametrize("seed", range(3))
def test_chosen_cost_not_below_best_static_subset(seed):
    """n <= 12: enumerate all 2^n static token subsets; the cheapest one reaching T is a
    lower bound for the cost of any static member of the family that reaches T."""
    n, d, T = 10, 4, 0.8
    Q, K, _, cls = rand_unit(60 + seed, n, d, bias=3.0)
    prof = fo.profile_unit(Q, K, cls, T, 0.2, 0.3, 0.5)
    colsum = fo.attention_map(Q, K, 0.5).sum(0)
    best = n
    for mask in range(1 << n):
        idx = [j for j in range(n) if mask >> j & 1]
        if colsum[idx].sum() / n >= T:
            best = min(best, len(idx))
    if prof.policy <= 2:
        assert prof.cost[prof.policy] >= best
    # and the family's static members reach T only with at least that many tokens
    for c in range(3):
        if prof.recovery[c] >= T:
            assert prof.cost[c] >= best


def test_cost_tie_prefers_smaller_policy_id():
    # no punctuation at all: |K_1| = |K_0| and R_1 = R_0 -> policy 0, not 1
    Q, K, _, cls = rand_unit(7, 30, 4, p_punct=0.0)
    K[:, 0] = 0
    K[0, 0] = 50
    Q[:, 0] = 1
    p = fo.profile_unit(Q, K, cls, 0.9, 0.3, 0.3, 1.0)
    assert p.cost[0] == p.cost[1] and p.policy == 0
    assert fo.select_policy(np.array([3, 3, 5, 9, 20]), np.array([.96, .96, .97, .99, 1.]), .95) == 0
    assert fo.select_policy(np.array([3, 4, 5, 9, 20]), np.array([.5, .96, .97, .99, 1.]), .95) == 1
    assert fo.select_policy(np.array([3, 4, 5, 9, 20]), np.array([.5, .6, .7, .8, 1.]), .95) == 4
    assert fo.select_policy(np.array([3, 4, 5, 9, 20]), np.array([.5, .6, .95, .99, 1.]), .95) == 2


def test_top_k_ties_and_full_sort():
    rng = np.random.default_rng(5)
    score = rng.integers(0, 6, size=40).astype(np.float64)   # many ties
    pos = rng.permutation(100)[:40]
    for k in [0, 1, 7, 39, 40, 55]:
        ref = sorted(sorted(range(40), key=lambda i: (-score[i], pos[i]))[:k], key=lambda i: pos[i])
        assert list(fo.top_k_positions(score, pos, k)) == [pos[i] for i in ref]
    assert fo.boundary_gap(np.array([4.0, 1.0, 2.0]), 1) == 0.5
    assert fo.boundary_gap(np.array([4.0, 1.0, 2.0]), 3) == math.inf


def test_budgets_floor_against_exact_rationals():
    for r, rs in [(0.1, "1/10"), (0.3, "3/10"), (0.25, "1/4")]:
        fr = Fraction(rs)
        for L in range(1, 20001):
            exact = (fr * L).numerator // (fr * L).denominator
            assert fo.frequent_budget(r, L) == exact, (r, L)
            assert fo.local_window(r, L) == max(1, exact), (r, L)


# ---------------------------------------------------------------- compaction and decode

def test_compaction_rows_identical_and_ascending():
    n, d = 40, 8
    Q, K, V, cls = rand_unit(70, n, d, bias=4.0)
    prof = fo.profile_unit(Q, K, cls, 0.9, 0.2, 0.2, 0.35)
    c = fo.compact_unit(K, V, cls, prof)
    assert np.all(np.diff(c.pos) > 0)
    assert c.pos.size == prof.cost[prof.policy]
    for slot, j in enumerate(c.pos):
        assert np.array_equal(c.K[slot], K[j]) and np.array_equal(c.V[slot], V[j])
        assert c.score[slot] == prof.colsum[j] and c.cls[slot] == cls[j]


def _decode_inputs(seed, S, d):
    rng = np.random.default_rng(seed)
    q, k, v = (rng.standard_normal((S, d)) for _ in range(3))
    cls = np.where(rng.random(S) < 0.2, 2, 0).astype(np.uint8)
    return q, k, v, cls


def test_full_policy_decode_is_dense_attention():
    n, d, S = 24, 8, 10
    Q, K, V, cls = rand_unit(80, n, d)
    q, k, v, cn = _decode_inputs(81, S, d)
    res = fo.run_unit(Q, K, V, cls, q, k, v, cn, 0.9, 0.3, 0.3, 0.4, forced_policy=4)
    assert res["profile"].recovery[4] == pytest.approx(1.0, abs=1e-14)
    for t in range(S):
        Kt = torch.from_numpy(np.vstack([K, k[: t + 1]]))
        Vt = torch.from_numpy(np.vstack([V, v[: t + 1]]))
        a = torch.softmax(Kt @ torch.from_numpy(q[t]) * 0.4, dim=0)
        assert np.allclose(res["outs"][t], (a @ Vt).numpy(), atol=1e-13)
        assert res["lens"][t] == n + t + 1


@pytest.mark.parametrize("policy", [0, 1])
def test_special_punct_decode_holds_only_those_classes(policy):
    n, d, S = 30, 8, 12
    Q, K, V, cls = rand_unit(82, n, d, p_punct=0.3)
    q, k, v, cn = _decode_inputs(83, S, d)
    res = fo.run_unit(Q, K, V, cls, q, k, v, cn, 0.9, 0.3, 0.3, 0.4, forced_policy=policy,
                      record_states=True)
    bits = 1 if policy == 0 else 3
    allcls = np.concatenate([cls, cn])
    allK, allV = np.vstack([K, k]), np.vstack([V, v])
    for t in range(S):
        expect = [j for j in range(n + t + 1) if allcls[j] & bits]
        assert list(res["states"][t]) == expect
        held = [j for j in range(n + t) if allcls[j] & bits] + [n + t]   # new token attends to itself
        lg = np.array([0.4 * q[t] @ allK[j] for j in held])
        a = np.exp(lg - lg.max())
        a /= a.sum()
        assert np.allclose(res["outs"][t], a @ allV[held], atol=1e-13)


def test_local_only_decode_is_sliding_window_attention():
    """policy 3 with r_f = 0 and no special/punct tokens: textbook windowed attention."""
    n, d, S = 30, 8, 15
    Q, K, V, _ = rand_unit(84, n, d)
    cls = np.zeros(n, dtype=np.uint8)
    q, k, v, _ = _decode_inputs(85, S, d)
    cn = np.zeros(S, dtype=np.uint8)
    r_l = 0.2
    w = 6
    res = fo.run_unit(Q, K, V, cls, q, k, v, cn, 0.9, r_l, 0.0, 0.4, forced_policy=3,
                      record_states=True)
    assert res["profile"].window == w
    assert list(res["init_pos"]) == list(range(n - w, n))
    allK, allV = np.vstack([K, k]), np.vstack([V, v])
    for t in range(S):
        p = n + t
        # held during the step: what the previous step kept (pos > p-1-w) plus the new token
        held = list(range(p - w, p + 1))
        lg = np.array([0.4 * q[t] @ allK[j] for j in held])
        a = np.exp(lg - lg.max())
        a /= a.sum()
        assert np.allclose(res["outs"][t], a @ allV[held], atol=1e-13)
        assert list(res["states"][t]) == list(range(p - w + 1, p + 1))


def test_q0_decode_scores_closed_form():
    """q = 0 at decode: a_j = 1/#held for every held token; scores follow exactly."""
    n, d, S = 20, 4, 8
    Q = np.zeros((n, d))
    K = np.ones((n, d))
    V = np.arange(n * d, dtype=np.float64).reshape(n, d)
    cls = np.zeros(n, dtype=np.uint8)
    cls[0] = 1
    q = np.zeros((S, d))
    k = np.ones((S, d))
    v = np.ones((S, d))
    cn = np.zeros(S, dtype=np.uint8)
    r_f = 0.5
    prof = fo.profile_unit(Q, K, cls, 0.5, 0.1, r_f, 1.0, forced_policy=2)
    cache = fo.compact_unit(K, V, cls, prof)
    assert list(cache.pos) == list(range(10))             # top 10 colsums = first 10 positions
    H = [harmonic(i) for i in range(n + 1)]
    score = {j: H[n] - H[j] for j in range(10)}
    for t in range(S):
        p = n + t
        o = fo.decode_step(cache, q[t], k[t], v[t], 0, t, 0.1, r_f, 1.0)
        held = sorted(score) + [p]
        score[p] = Fraction(0)
        for j in held:
            score[j] += Fraction(1, len(held))
        assert np.allclose(o, np.mean(np.vstack([V, v])[held], axis=0), atol=1e-12)
        kf = (p + 1) // 2
        ranked = sorted(held, key=lambda j: (-score[j], j))
        keep = set(ranked[:kf]) | {0}
        score = {j: s for j, s in score.items() if j in keep}
        assert list(cache.pos) == sorted(keep)
        assert np.allclose(cache.score, [float(score[j]) for j in sorted(keep)], atol=1e-13)


@pytest.mark.parametrize("policy", [2, 3])
def test_decode_set_equation_rederived_each_step(policy):
    """Independent re-derivation with python sets/dicts (no shared helper): held and scores
    after every step for the policies that contain `frequent`."""
    n, d, S = 26, 8, 20
    scale, r_l, r_f = 0.4, 0.2, 0.3
    Q, K, V, cls = rand_unit(90 + policy, n, d, p_punct=0.15)
    q, k, v, cn = _decode_inputs(95, S, d)
    res = fo.run_unit(Q, K, V, cls, q, k, v, cn, 0.9, r_l, r_f, scale, forced_policy=policy,
                      record_states=True)
    prof = res["profile"]
    w = max(1, math.floor(r_l * n))
    allK, allV, allc = np.vstack([K, k]), np.vstack([V, v]), np.concatenate([cls, cn])
    score = {int(j): float(prof.colsum[j]) for j in res["init_pos"]}
    for t in range(S):
        p = n + t
        score[p] = 0.0
        held = sorted(score)
        lg = np.array([scale * q[t] @ allK[j] for j in held])
        a = np.exp(lg - lg.max())
        a /= a.sum()
        assert np.allclose(res["outs"][t], a @ allV[held], atol=1e-12)
        for j, aj in zip(held, a):
            score[j] += aj
        kf = math.floor(r_f * (p + 1))
        ranked = sorted(held, key=lambda j: (-score[j], j))
        keep = set(ranked[:kf]) | {j for j in held if allc[j] & 3}
        if policy == 3:
            keep |= {j for j in held if j > p - w}
        score = {j: s for j, s in score.items() if j in keep}
        assert list(res["states"][t]) == sorted(keep)


# ------------------------------------- other policy tables (App. A.1 Tables 4-5, Sec. 5.1)

FAMILIES = [
    (8, 8 | 4, 8 | 4 | 1, 15),   # components added in another order: local first
    (1, 1 | 2, 1 | 2 | 8, 15),   # local before frequent
    (1, 1 | 4, 1 | 4 | 8, 0),    # punctuation left out, one id unused
    (4, 8, 4 | 8, 0),            # the fixed baselines: frequent, local, frequent+local
    (2, 4, 8, 1),                # single components, not nested
]


def _letters(mask):
    return "".join(ch for bit, ch in ((1, "s"), (2, "p"), (4, "f"), (8, "l")) if mask & bit)


@pytest.mark.parametrize("fam", range(len(FAMILIES)))
@pytest.mark.parametrize("seed", range(3))
def test_family_tables_match_brute_force(seed, fam):
    """Cost and recovery of every member of an arbitrary table, and the literal argmin of
    Eq. 1 over its usable members, by loops over the dense map."""
    family = FAMILIES[fam]
    n, d = 18, 4
    T = [0.7, 0.85, 0.95][seed]
    Q, K, _, cls = rand_unit(300 + 7 * seed + fam, n, d, p_punct=0.2, bias=[0.0, 3.0, 6.0][seed])
    scale, r_l, r_f = 0.5, 0.25, 0.2
    prof = fo.profile_unit(Q, K, cls, T, r_l, r_f, scale, family=family)
    A = fo.attention_map(Q, K, scale)
    w, k = max(1, math.floor(r_l * n)), math.floor(r_f * n)
    colsum = A.sum(0)
    ranked = sorted(range(n), key=lambda j: (-colsum[j], j))
    base = {"s": {j for j in range(n) if cls[j] & 1}, "p": {j for j in range(n) if cls[j] & 2},
            "f": set(ranked[:k])}
    cands = [(n, 4)]
    for c, mask in enumerate(family):
        if mask == 0:
            continue
        combo = _letters(mask)
        static = set().union(*[base[x] for x in combo if x != "l"]) if combo.strip("l") else set()
        end_set = static | (set(range(n - w, n)) if "l" in combo else set())
        rec = 0.0
        for i in range(n):
            cols = {j for j in static if j <= i}
            if "l" in combo:
                cols |= set(range(max(0, i - w + 1), i + 1))
            rec += sum(A[i, j] for j in cols)
        rec /= n
        assert prof.cost[c] == len(end_set)
        assert abs(prof.recovery[c] - rec) < 1e-13
        assert sorted(prof.sets[c]) == sorted(end_set)
        if rec >= T:
            cands.append((len(end_set), c))
    assert prof.policy == min(cands)[1]
    assert family[prof.policy] != 0 if prof.policy < 4 else True


def test_default_family_is_eq2_and_unused_ids_never_chosen():
    assert fo.DEFAULT_FAMILY == (1, 3, 7, 15)
    Q, K, _, cls = rand_unit(11, 24, 4, bias=9.0)
    a = fo.profile_unit(Q, K, cls, 0.5, 0.3, 0.3, 1.0)
    b = fo.profile_unit(Q, K, cls, 0.5, 0.3, 0.3, 1.0, family=(1, 3, 7, 15))
    assert a.policy == b.policy and np.array_equal(a.recovery, b.recovery)
    # T below every recovery: the cheapest usable member wins, never the empty id 0
    c = fo.profile_unit(Q, K, cls, 1e-9, 0.3, 0.3, 1.0, family=(0, 8, 0, 15))
    assert c.policy == 1


@pytest.mark.parametrize("mask", [4, 8, 4 | 8, 1 | 8, 2 | 4])
def test_family_decode_set_equation_rederived_each_step(mask):
    """A forced single-table member: held set, scores and outputs after every step re-derived
    with python sets (frequent = fixed-ratio heavy hitters, local = sliding window)."""
    n, d, S = 22, 8, 18
    scale, r_l, r_f = 0.4, 0.2, 0.3
    family = (mask, 0, 0, 0)
    Q, K, V, cls = rand_unit(400 + mask, n, d, p_punct=0.2)
    q, k, v, cn = _decode_inputs(410 + mask, S, d)
    res = fo.run_unit(Q, K, V, cls, q, k, v, cn, 0.9, r_l, r_f, scale, forced_policy=0,
                      record_states=True, family=family)
    prof = res["profile"]
    w = max(1, math.floor(r_l * n))
    allK, allV, allc = np.vstack([K, k]), np.vstack([V, v]), np.concatenate([cls, cn])
    score = {int(j): float(prof.colsum[j]) for j in res["init_pos"]}
    cbits = mask & 3
    for t in range(S):
        p = n + t
        score[p] = 0.0
        held = sorted(score)
        lg = np.array([scale * q[t] @ allK[j] for j in held])
        a = np.exp(lg - lg.max())
        a /= a.sum()
        assert np.allclose(res["outs"][t], a @ allV[held], atol=1e-12)
        keep = {j for j in held if allc[j] & cbits}
        if mask & 4:
            for j, aj in zip(held, a):
                score[j] += aj
            ranked = sorted(held, key=lambda j: (-score[j], j))
            keep |= set(ranked[:math.floor(r_f * (p + 1))])
        if mask & 8:
            keep |= {j for j in held if j > p - w}
        score = {j: s for j, s in score.items() if j in keep}
        assert list(res["states"][t]) == sorted(keep)


# ----------------------------------------- stability probe at decode steps (Sec. 4, Fig. 4)

@pytest.mark.parametrize("policy", [4, 3, 1])
def test_step_recovery_rederived_with_sets(policy):
    """Per decode step: mass of the new token's attention row on special / +punct / +frequent /
    +local tokens among the held ones, from python dicts. With the full cache (policy 4) this is
    the row's recovery under every member of Eq. 2's family; the members are nested, the last
    entry is the whole row."""
    n, d, S = 24, 8, 16
    scale, r_l, r_f = 0.4, 0.2, 0.3
    Q, K, V, cls = rand_unit(500 + policy, n, d, p_punct=0.2)
    q, k, v, cn = _decode_inputs(510 + policy, S, d)
    res = fo.run_unit(Q, K, V, cls, q, k, v, cn, 0.9, r_l, r_f, scale, forced_policy=policy,
                      record_states=True, probe=True)
    prof = res["profile"]
    w = max(1, math.floor(r_l * n))
    allK, allc = np.vstack([K, k]), np.concatenate([cls, cn])
    score = {int(j): float(prof.colsum[j]) for j in res["init_pos"]}
    for t in range(S):
        p = n + t
        score[p] = 0.0
        held = sorted(score)
        lg = np.array([scale * q[t] @ allK[j] for j in held])
        a = np.exp(lg - lg.max())
        a /= a.sum()
        att = dict(zip(held, a))
        for j in held:
            score[j] += att[j]      # probing keeps the cumulative score for every policy
        ranked = sorted(held, key=lambda j: (-score[j], j))
        sets = [{j for j in held if allc[j] & 1}]
        sets.append(sets[0] | {j for j in held if allc[j] & 2})
        sets.append(sets[1] | set(ranked[:math.floor(r_f * (p + 1))]))
        sets.append(sets[2] | {j for j in held if j > p - w})
        rho = res["probes"][t]
        for c in range(4):
            assert abs(rho[c] - sum(att[j] for j in sets[c])) < 1e-13
        assert abs(rho[4] - 1.0) < 1e-13 and np.all(np.diff(rho) >= -1e-15)
        keep = set(res["states"][t])
        score = {j: s for j, s in score.items() if j in keep}
    # probing does not change what is kept or computed
    ref = fo.run_unit(Q, K, V, cls, q, k, v, cn, 0.9, r_l, r_f, scale, forced_policy=policy,
                      record_states=True)
    assert np.array_equal(ref["outs"], res["outs"])
    assert all(np.array_equal(x, y) for x, y in zip(ref["states"], res["states"]))


# ------------------------------------ grouped query heads sharing one K/V head (reading R13)

def test_group_of_identical_heads_equals_one_head():
    """G copies of one query head: same recoveries, policy and kept sets, G-fold scores, and
    every head's decode output equals the single-head output."""
    n, d, S, G = 28, 8, 14, 3
    scale, r_l, r_f = 0.4, 0.2, 0.3
    Q, K, V, cls = rand_unit(600, n, d, p_punct=0.2, bias=2.0)
    q, k, v, cn = _decode_inputs(601, S, d)
    for policy in (-1, 2, 3):
        one = fo.run_unit(Q, K, V, cls, q, k, v, cn, 0.9, r_l, r_f, scale, forced_policy=policy,
                          record_states=True)
        grp = fo.run_unit(np.stack([Q] * G), K, V, cls, np.stack([q] * G, axis=1), k, v, cn, 0.9, r_l, r_f,
                          scale, forced_policy=policy, record_states=True)
        assert grp["profile"].policy == one["profile"].policy
        assert np.allclose(grp["profile"].recovery, one["profile"].recovery, atol=1e-14)
        assert np.allclose(grp["profile"].colsum, G * one["profile"].colsum, rtol=1e-14)
        for t in range(S):
            assert np.array_equal(grp["states"][t], one["states"][t])
            for g in range(G):
                assert np.allclose(grp["outs"][t][g], one["outs"][t], atol=1e-13)
            assert np.allclose(grp["score_states"][t], G * one["score_states"][t], rtol=1e-12)


@pytest.mark.parametrize("policy", [2, 3])
def test_group_of_two_heads_rederived_by_loops(policy):
    """G = 2 different query heads: recoveries as the mean over the 2n rows, scores as the sum of
    both heads' attention, one shared kept set -- by loops and python sets."""
    n, d, S, G = 20, 6, 12, 2
    scale, r_l, r_f = 0.5, 0.25, 0.3
    Q0, K, V, cls = rand_unit(610 + policy, n, d, p_punct=0.2, bias=1.5)
    Q1 = np.random.default_rng(620 + policy).standard_normal((n, d))
    rng = np.random.default_rng(630 + policy)
    q = rng.standard_normal((S, G, d))
    _, k, v, cn = _decode_inputs(640 + policy, S, d)
    res = fo.run_unit(np.stack([Q0, Q1]), K, V, cls, q, k, v, cn, 0.9, r_l, r_f, scale,
                      forced_policy=policy, record_states=True)
    prof = res["profile"]
    A = [fo.attention_map(Q0, K, scale), fo.attention_map(Q1, K, scale)]
    w, kf = max(1, math.floor(r_l * n)), math.floor(r_f * n)
    colsum = [sum(A[g][i, j] for g in range(G) for i in range(n)) for j in range(n)]
    assert np.allclose(prof.colsum, colsum, atol=1e-13)
    ranked = sorted(range(n), key=lambda j: (-colsum[j], j))
    static = {j for j in range(n) if cls[j] & 3} | set(ranked[:kf])
    rec2 = sum(A[g][i, j] for g in range(G) for i in range(n) for j in static if j <= i) / (G * n)
    assert abs(prof.recovery[2] - rec2) < 1e-13
    rec3 = 0.0
    for g in range(G):
        for i in range(n):
            cols = {j for j in static if j <= i} | set(range(max(0, i - w + 1), i + 1))
            rec3 += sum(A[g][i, j] for j in cols)
    assert abs(prof.recovery[3] - rec3 / (G * n)) < 1e-13
    # decode: one kept set, G outputs, scores += both rows
    allK, allV, allc = np.vstack([K, k]), np.vstack([V, v]), np.concatenate([cls, cn])
    score = {int(j): float(colsum[j]) for j in res["init_pos"]}
    for t in range(S):
        p = n + t
        score[p] = 0.0
        held = sorted(score)
        for g in range(G):
            lg = np.array([scale * q[t, g] @ allK[j] for j in held])
            a = np.exp(lg - lg.max())
            a /= a.sum()
            assert np.allclose(res["outs"][t][g], a @ allV[held], atol=1e-12)
            for j, aj in zip(held, a):
                score[j] += aj
        rk = sorted(held, key=lambda j: (-score[j], j))
        keep = set(rk[:math.floor(r_f * (p + 1))]) | {j for j in held if allc[j] & 3}
        if policy == 3:
            keep |= {j for j in held if j > p - w}
        score = {j: s for j, s in score.items() if j in keep}
        assert list(res["states"][t]) == sorted(keep)


# ---------------------------------------------------------------- token classes (Sec. 3.4)

def test_classify_tokens_by_hand_and_against_set_membership():
    ids = np.array([[0, 5, 7, 5, 9], [13, 0, 2, 7, 7]])
    got = fo.classify_tokens(ids, special_ids=[0, 7], punct_ids=[5, 7, 13])
    # 0 -> special; 5, 13 -> punctuation; 7 is in both lists -> both bits; 9, 2 -> nothing
    assert got.tolist() == [[1, 2, 3, 2, 0], [2, 1, 0, 3, 3]] and got.dtype == np.uint8
    assert fo.classify_tokens(ids, [], []).tolist() == [[0] * 5, [0] * 5]
    rng = np.random.default_rng(5)
    big = rng.integers(0, 50, size=(3, 200))
    sp, pu = [1, 2, 3], [3, 10, 20, 30]
    ref = np.isin(big, sp).astype(np.uint8) | (np.isin(big, pu).astype(np.uint8) << 1)
    assert np.array_equal(fo.classify_tokens(big, sp, pu), ref)
