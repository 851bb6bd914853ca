"""Pins for the oracle's replica plan and dispatch (CPU only).

What fixes the expected values: the scenario the paper prints (tests/golden), Algorithm 1's
closed form at slot capacity 1, the invariants stated in the "Capacity capping" subsection,
and a separately written token-by-token walk (oracle/brute_force.py).
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import brute_force as bf


def _golden(golden_dir):
    kv = {}
    with open(os.path.join(golden_dir, "replication_scenario.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            kv[k] = int(v)
    return kv


def test_paper_scenario_two_active_experts(golden_dir):
    g = _golden(golden_dir)
    T, E = g["batch_tokens"], g["experts"]
    rng = np.random.default_rng(5)
    a, b = 17, 40
    ids = np.array([a] * g["tokens_per_active_expert"] + [b] * (T - g["tokens_per_active_expert"]),
                   np.int32)
    rng.shuffle(ids)
    for policy in (0, 1):
        p = oracle.plan(ids, E, R=T - g["active_experts"], C_=g["tokens_per_physical_replica"],
                        policy=policy)
        assert p["replicas"][a] == g["replicas_per_active_expert"]
        assert p["replicas"][b] == g["replicas_per_active_expert"]
        others = np.delete(p["replicas"], [a, b])
        assert (others == 1).all()
        x = rng.standard_normal((T, 4)).astype(np.float32)
        d = oracle.dispatch(x, ids, p["replicas"], E, 1, E + T)
        assert d["kept"].sum() == T and (d["inv"] >= 0).all()        # nobody waits / drops
        sizes = np.diff(d["slot_offset"][: p["n_slots"] + 1])
        own = sizes[p["slot_base"][a]: p["slot_base"][a + 1]]
        assert (own == 1).all() and own.size == 32                    # one token per replica
        assert sizes.max() == 1


@pytest.mark.parametrize("seed", range(5))
def test_algorithm1_uncapped_closed_form(seed):
    rng = np.random.default_rng(seed)
    E, T = 12, 90
    ids = rng.choice(E, size=T, p=rng.dirichlet(np.ones(E) * 0.3)).astype(np.int32)
    p = oracle.plan(ids, E, R=10 * T, C_=1)
    n = np.bincount(ids, minlength=E)
    assert (p["replicas"] == np.maximum(1, n)).all()
    assert (p["counts"] == n).all()


def _check_plan_invariants(ids, E, R, C, policy, p):
    n = np.bincount(ids, minlength=E)
    want = np.maximum(0, -(-n // C) - 1)
    r = p["replicas"]
    assert (r >= 1).all()
    assert (r - 1).sum() <= R
    assert ((r - 1) <= want).all()
    if want.sum() <= R:
        assert (r == 1 + want).all()
    else:
        assert (r - 1).sum() == R          # an over-subscribed budget is used in full
    assert p["n_slots"] == r.sum()
    assert (np.diff(p["slot_base"]) == r).all() and p["slot_base"][0] == 0
    se = p["slot_expert"][: p["n_slots"]]
    assert (se == np.repeat(np.arange(E), r)).all()


@pytest.mark.parametrize("policy", [0, 1])
def test_plan_invariants_and_brute_force(policy):
    rng = np.random.default_rng(100 + policy)
    for trial in range(200):
        E = int(rng.integers(1, 9))
        T = int(rng.integers(0, 70))
        C = int(rng.integers(1, 9))
        R = int(rng.integers(0, 12))
        ids = rng.choice(E, size=T, p=rng.dirichlet(np.ones(E) * 0.5)).astype(np.int32)
        p = oracle.plan(ids, E, R, C, policy)
        _check_plan_invariants(ids, E, R, C, policy, p)
        assert list(p["replicas"]) == bf.plan(ids, E, R, C, policy), (trial, E, T, C, R)


def test_wants_from_token_walk_equal_ceiling_formula():
    rng = np.random.default_rng(3)
    for _ in range(100):
        E, C = int(rng.integers(1, 6)), int(rng.integers(1, 7))
        ids = rng.integers(0, E, size=int(rng.integers(0, 60)))
        n = np.bincount(ids, minlength=E)
        assert bf.wants_by_token_walk([int(i) for i in ids], E, C) == \
            list(np.maximum(0, -(-n // C) - 1))


def test_proportional_policy_hand_case():
    # n = (50, 30, 10, 4), C = 10: wants (4, 2, 0, 0), D = 6.  R = 3 < D.
    # floor(3*4/6) = 2, floor(3*2/6) = 1 -> all three granted by the floors.
    ids = np.repeat(np.arange(4), [50, 30, 10, 4]).astype(np.int32)
    assert list(oracle.plan(ids, 4, 3, 10, 0)["replicas"]) == [3, 2, 1, 1]
    # R = 4: floors 2 and 1 (sum 3); one left -> loads per slot 50/3 = 16.7 vs 30/2 = 15 -> e0.
    assert list(oracle.plan(ids, 4, 4, 10, 0)["replicas"]) == [4, 2, 1, 1]
    # R = 5: floors floor(20/6)=3, floor(10/6)=1; one left -> 50/4 = 12.5 vs 30/2 = 15 -> e1.
    assert list(oracle.plan(ids, 4, 5, 10, 0)["replicas"]) == [4, 3, 1, 1]
    # equal-share reading: R = 3, two wanting experts -> 1 each, then the last one by load:
    # 50/2 = 25 vs 30/2 = 15 -> e0.
    assert list(oracle.plan(ids, 4, 3, 10, 1)["replicas"]) == [3, 2, 1, 1]
    # R = 2: one each, nothing left.
    assert list(oracle.plan(ids, 4, 2, 10, 1)["replicas"]) == [2, 2, 1, 1]


def test_proportional_policy_r2_hand_case():
    # R = 2: floors floor(8/6)=1, floor(4/6)=0; one left: 50/2 = 25 vs 30/1 = 30 -> e1.
    ids = np.repeat(np.arange(4), [50, 30, 10, 4]).astype(np.int32)
    assert list(oracle.plan(ids, 4, 2, 10, 0)["replicas"]) == [2, 2, 1, 1]


def test_tie_break_lowest_id():
    ids = np.repeat(np.arange(3), [30, 30, 30]).astype(np.int32)   # wants 2,2,2; D=6
    # R = 4: floors floor(8/6) = 1 each (3 used); one left, equal loads 30/2 -> lowest id.
    assert list(oracle.plan(ids, 3, 4, 10, 0)["replicas"]) == [3, 2, 2]


def test_plan_rejects_bad_arguments():
    ids = np.array([0, 1, 5], np.int32)
    with pytest.raises(ValueError):
        oracle.plan(ids, 4, 1, 1)           # id out of range
    with pytest.raises(ValueError):
        oracle.plan(ids[:2], 4, -1, 1)
    with pytest.raises(ValueError):
        oracle.plan(ids[:2], 4, 1, 0)


# ------------------------------------------------------------------ dispatch
def _check_dispatch(ids, rep, E, C, dsp, x):
    T = ids.shape[0]
    r = np.ones(E, np.int64) if rep is None else rep.astype(np.int64)
    n = np.bincount(ids, minlength=E)
    assert (dsp["counts"] == n).all()
    assert (dsp["kept"] == np.minimum(n, r * C)).all()
    K = int(dsp["kept"].sum())
    assert dsp["expert_offset"][0] == 0 and dsp["expert_offset"][E] == K
    assert (np.diff(dsp["expert_offset"]) == dsp["kept"]).all()
    perm, inv = dsp["perm"], dsp["inv"]
    assert K + int((inv < 0).sum()) == T                       # conservation
    assert sorted(perm[:K]) == sorted(np.nonzero(inv >= 0)[0])  # bijection onto kept tokens
    assert (inv[perm[:K]] == np.arange(K)).all()
    assert (perm[K:] == -1).all()
    e_along = ids[perm[:K]]
    assert (np.diff(e_along) >= 0).all()                       # expert-sorted
    same = np.diff(e_along) == 0
    assert (np.diff(perm[:K])[same] > 0).all()                 # stable inside an expert
    # dropped tokens are exactly the late ones
    for e in range(E):
        toks = np.nonzero(ids == e)[0]
        assert (inv[toks[: dsp["kept"][e]]] >= 0).all() and (inv[toks[dsp["kept"][e]:]] < 0).all()
    P = int(r.sum())
    so = dsp["slot_offset"]
    assert (so[P:] == K).all()
    sizes = np.diff(so[: P + 1])
    assert sizes.min(initial=0) >= 0 and sizes.max(initial=0) <= C
    base = np.concatenate([[0], np.cumsum(r)])
    for e in range(E):
        assert so[base[e]] == dsp["expert_offset"][e]          # refinement of expert ranges
        own = sizes[base[e]: base[e + 1]]
        assert own.sum() == dsp["kept"][e]
        assert own.max() - own.min() <= 1 and (np.diff(own) <= 0).all()
    assert (dsp["x_perm"][:K] == x[perm[:K]]).all()


def test_dispatch_invariants_random():
    rng = np.random.default_rng(11)
    for trial in range(150):
        E = int(rng.integers(1, 10))
        T = int(rng.integers(0, 120))
        C = int(rng.integers(1, 12))
        R = int(rng.integers(0, 8))
        ids = rng.choice(E, size=T, p=rng.dirichlet(np.ones(E) * 0.4)).astype(np.int32)
        x = rng.standard_normal((T, 3)).astype(np.float32)
        rep = None if trial % 5 == 0 else oracle.plan(ids, E, R, C, trial % 2)["replicas"]
        dsp = oracle.dispatch(x, ids, rep, E, C, E + R)
        _check_dispatch(ids, rep, E, C, dsp, x)


def test_dispatch_matches_quadratic_rank():
    rng = np.random.default_rng(12)
    E, T, C = 5, 80, 7
    ids = rng.integers(0, E, size=T).astype(np.int32)
    rep = np.array([1, 2, 1, 3, 1], np.int32)
    x = rng.standard_normal((T, 2)).astype(np.float32)
    dsp = oracle.dispatch(x, ids, rep, E, C, 10)
    for s in range(T):
        j = sum(1 for t in range(s) if ids[t] == ids[s])
        if j < rep[ids[s]] * C:
            before = sum(min(int((ids == e).sum()), int(rep[e]) * C) for e in range(ids[s]))
            assert dsp["inv"][s] == before + j
        else:
            assert dsp["inv"][s] == -1


def test_plan_from_exact_counts_never_drops_when_budget_suffices():
    rng = np.random.default_rng(13)
    for _ in range(50):
        E, C = 6, int(rng.integers(2, 9))
        ids = rng.choice(E, size=60, p=rng.dirichlet(np.ones(E) * 0.3)).astype(np.int32)
        n = np.bincount(ids, minlength=E)
        D = int(np.maximum(0, -(-n // C) - 1).sum())
        p = oracle.plan(ids, E, D, C)
        x = np.zeros((60, 1), np.float32)
        dsp = oracle.dispatch(x, ids, p["replicas"], E, C, E + D)
        assert (dsp["inv"] >= 0).all()


def test_monotone_in_budget_small_exhaustive():
    """Policy 0 on a small exhaustive grid: raising the budget never lowers an expert's slot count
    (checked, not assumed: the proportional floors are re-derived at each R)."""
    bad = []
    for n in itertools.product([0, 3, 7, 12, 20], repeat=3):
        ids = np.repeat(np.arange(3), n).astype(np.int32)
        prev = None
        for R in range(0, 12):
            r = oracle.plan(ids, 3, R, 4, 0)["replicas"]
            if prev is not None and (r < prev).any():
                bad.append((n, R))
            prev = r
    assert bad == []


def test_budget_monotonicity_is_not_a_law():
    """The property above is not general: floors of proportional shares plus a largest-load remainder can
    take a slot from one expert when the budget grows by one (the apportionment paradox).  One such case,
    found by random search (2 in 3000 for policy 0), is kept here with the hand-checked shares so that the
    text of the design notes stays honest about it."""
    n = [16, 15, 15, 14, 24, 25, 26, 31]
    ids = np.repeat(np.arange(8), n).astype(np.int32)
    # C = 8: wants = ceil(n/8) - 1 = [1,1,1,1,2,3,3,3], D = 15
    r9 = oracle.plan(ids, 8, 9, 8, 0)["replicas"]
    r10 = oracle.plan(ids, 8, 10, 8, 0)["replicas"]
    # R = 9: floors 9*w/15 = [0,0,0,0,1,1,1,1], five slots left, handed out by load per slot
    # R = 10: floors 10*w/15 = [0,0,0,0,1,2,2,2], three slots left
    assert r9.sum() == 8 + 9 and r10.sum() == 8 + 10
    assert r9.tolist() == [2, 2, 2, 2, 2, 2, 2, 3]
    assert r10.tolist() == [2, 2, 2, 1, 2, 3, 3, 3]
    assert (r10 < r9).any()
