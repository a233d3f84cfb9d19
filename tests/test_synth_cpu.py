"""The seeded input generators: deterministic, of the stated shapes and class statistics, and
planting the attention structures they claim to plant (judged by the float64 oracle)."""
import numpy as np
import torch

from oracle import fastgen_oracle as fo
from paper_2310_01801_amd import synth

W = synth.WORKLOADS


def _small(**kw):
    base = dict(name="synth", layers=2, heads=10, batch=2, prompt_len=192, steps=12, seed=5)
    base.update(kw)
    return W["llama7b_b1"].scaled(**base)


def test_generators_are_deterministic_and_typed():
    w = _small()
    plan = synth.unit_plan(w)
    cp, cd = synth.token_classes(w)
    a = synth.prompt_unit(w, plan, cp, 7)
    b = synth.prompt_unit(w, plan, cp, 7)
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    assert all(x.dtype == torch.bfloat16 and tuple(x.shape) == (192, 128) for x in a)
    assert not torch.equal(a[0], synth.prompt_unit(w, plan, cp, 8)[0])
    q = synth.decode_unit(w, plan, cd, 7)
    assert all(tuple(x.shape) == (12, 128) for x in q)
    Q, K, V = synth.prompt_batch(w, plan, cp, [3, 7])
    assert torch.equal(Q[1], a[0]) and torch.equal(K[1], a[1]) and torch.equal(V[1], a[2])
    # another seed gives other inputs
    w2 = _small(seed=6)
    assert not torch.equal(synth.prompt_unit(w2, synth.unit_plan(w2), synth.token_classes(w2)[0], 7)[0], a[0])


def test_token_classes_follow_the_recipe():
    w = _small(prompt_len=4000, batch=4)
    cp, cd = synth.token_classes(w)
    assert cp.shape == (4, 4000) and cd.shape == (12, 4)
    assert np.all(cp[:, 0] & synth.CLASS_SPECIAL) and not np.any(cp[:, 1:] & synth.CLASS_SPECIAL)
    frac = np.mean((cp[:, 1:] & synth.CLASS_PUNCT) != 0)
    assert 0.05 < frac < 0.2          # punctuation: about one token in ten
    assert not np.any(cd & synth.CLASS_SPECIAL)   # no new special tokens while decoding


def test_planted_patterns_show_up_in_the_oracle_profile():
    """Each planted pattern is recovered by the policy it is meant to favour: the recipe gives
    the workload its spread over the five policies."""
    w = _small(prompt_len=256, layers=4, heads=10)
    plan = synth.unit_plan(w)
    cp, _ = synth.token_classes(w)
    scale = 1.0 / np.sqrt(w.head_dim)
    seen = set()
    for u in range(w.num_units):
        pat = int(plan.pattern[u])
        if pat in seen or float(plan.strength[u]) < 3.0 and pat != synth.BROAD:
            continue
        seen.add(pat)
        Q, K, _ = synth.prompt_unit(w, plan, cp, u)
        p = fo.profile_unit(synth.to_f64(Q), synth.to_f64(K), cp[u // w.units_per_seq], 0.95, 0.3, 0.3, scale)
        R = p.recovery
        if pat == synth.SPECIAL:
            assert R[0] > 0.8                       # mass on the special token
        elif pat == synth.PUNCT:
            assert R[1] > 0.8 and R[1] > R[0] + 0.2  # mass on special + punctuation
        elif pat == synth.HEAVY:
            assert R[2] > R[1] + 0.2                # heavy hitters: the frequent policy recovers it
        elif pat == synth.LOCAL:
            assert R[3] > R[2] + 0.2                # only the window does
        else:
            assert R[3] < 0.95 and p.policy == 4     # broad: nothing short of the full cache
    assert seen == {synth.LOCAL, synth.SPECIAL, synth.PUNCT, synth.HEAVY, synth.BROAD}


def test_grouped_query_heads_share_the_planted_dimensions():
    w = _small()
    plan = synth.unit_plan(w)
    cp, cd = synth.token_classes(w)
    u = int(np.nonzero(plan.pattern == synth.SPECIAL)[0][0])
    Qg = synth.prompt_group_queries(w, plan, cp, u, 3)
    assert tuple(Qg.shape) == (3, 192, 128)
    assert torch.equal(Qg[0], synth.prompt_unit(w, plan, cp, u)[0])
    assert torch.equal(Qg[0][:, 0], Qg[1][:, 0]) and not torch.equal(Qg[0][:, 5], Qg[1][:, 5])
    qg = synth.decode_group_queries(w, plan, cd, u, 3)
    assert tuple(qg.shape) == (12, 3, 128) and torch.equal(qg[:, 0], synth.decode_unit(w, plan, cd, u)[0])
