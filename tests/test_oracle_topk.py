"""Pins for the oracle's top-k routing (CPU only): ``oracle/topk.py`` and its wrappers.

Independent anchors: numpy's stable sort and scipy's softmax for the selection, closed forms
(a geometric gate, equal logits), the top-1 oracle in C for k = 1, torch's bfloat16 conversion
for the storage rounding, and a per-assignment walk written out in this file for the whole layer.
"""
import numpy as np
import pytest
import torch
from scipy.special import softmax as scipy_softmax

import oracle
import synth
from oracle import topk


def _logits(T, E, seed, scale=2.0):
    return np.random.default_rng(seed).standard_normal((T, E)) * scale


# ------------------------------------------------------------------ selection
@pytest.mark.parametrize("k", [1, 2, 3, 5])
def test_select_matches_stable_sort_and_library_softmax(k):
    l = _logits(200, 11, 3)
    l[::7, 4] = l[::7, 9]                                  # some exact ties
    sel = topk.select(l, k)
    order = np.argsort(-l, axis=1, kind="stable")[:, :k]   # descending, lower id first among equals
    assert (sel["idx"].T == order).all()
    p = scipy_softmax(l, axis=1)
    assert np.allclose(sel["weight"].T, np.take_along_axis(p, order, 1), rtol=1e-12, atol=0)
    srt = -np.sort(-l, axis=1)
    want_gap = (srt[:, :k] - srt[:, 1:k + 1]).min(axis=1)
    assert np.allclose(sel["gap"], want_gap, atol=1e-12)
    assert (sel["gap"][::7] >= 0).all()


def test_select_geometric_gate_closed_form():
    E, k, c = 9, 3, 0.75
    l = np.tile(np.arange(E) * c, (4, 1))                  # logit e*c: p_e = r^(E-1-e) (1-r)/(1-r^E)
    sel = topk.select(l, k)
    assert (sel["idx"] == np.array([[E - 1], [E - 2], [E - 3]])).all()
    r = np.exp(-c)
    want = r ** np.arange(k) * (1 - r) / (1 - r ** E)
    assert np.allclose(sel["weight"], want[:, None], rtol=1e-12)
    assert np.allclose(sel["gap"], c)
    ren = topk.select(l, k, renormalize=True)
    assert np.allclose(ren["weight"], (r ** np.arange(k) / (1 + r + r * r))[:, None], rtol=1e-12)


def test_select_equal_logits_lowest_ids_uniform_weights():
    sel = topk.select(np.zeros((3, 6)), 4)
    assert (sel["idx"] == np.arange(4)[:, None]).all()
    assert np.allclose(sel["weight"], 1 / 6)
    assert (sel["gap"] == 0).all()
    assert np.allclose(topk.select(np.zeros((3, 6)), 4, True)["weight"], 0.25)


def test_select_weight_sums_and_expert_permutation():
    l = _logits(64, 8, 5)
    for k in (1, 3, 8):
        s = topk.select(l, k)
        tot = s["weight"].sum(axis=0)
        assert (tot <= 1 + 1e-12).all() and (np.allclose(tot, 1) == (k == 8))
        assert np.allclose(topk.select(l, k, True)["weight"].sum(axis=0), 1, rtol=1e-12)
        assert (np.diff(s["weight"], axis=0) <= 0).all()        # choices come in descending order
    pi = np.random.default_rng(6).permutation(8)                # expert e moves to column pi[e]
    lp = np.empty_like(l)
    lp[:, pi] = l
    a, b = topk.select(l, 3), topk.select(lp, 3)
    assert (pi[a["idx"]] == b["idx"]).all() and np.allclose(a["weight"], b["weight"], rtol=1e-12)


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_route_topk_first_choice_is_the_top1_router(dtype):
    c = synth.moe_layer_inputs(96, 16, 8, 12, dtype, 1.0, 21)
    r1 = oracle.route(c["x"], c["w_router"], c["b_router"])
    rk = oracle.route_topk(c["x"], c["w_router"], c["b_router"], 3)
    assert (rk["idx"][0] == r1["idx"]).all()
    assert np.allclose(rk["weight"][0], r1["prob"], rtol=2e-7)
    assert (rk["idx"][1] == r1["idx2"]).all()
    # the k ids of a token are distinct
    srt = np.sort(rk["idx"], axis=0)
    assert (np.diff(srt, axis=0) > 0).all()


# ------------------------------------------------------------------ combine
def _combine_case(dtype, k=3, T=40, d=8, rows=70, seed=9):
    rng = np.random.default_rng(seed)
    x = synth.normal_tensor((T, d), 1.0, [seed, 1], dtype)
    y = synth.normal_tensor((rows, d), 1.0, [seed, 2], dtype)
    inv = np.full(k * T, -1, np.int32)
    kept = rng.permutation(k * T)[:rows]
    inv[kept] = rng.permutation(rows).astype(np.int32)
    inv = inv.reshape(k, T)
    inv[:, 5] = -1                                           # a token with no kept choice
    w = rng.random((k, T)).astype(np.float32)
    return x, y, inv, w


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
@pytest.mark.parametrize("residual", [0, 1])
def test_combine_topk_per_element_walk(dtype, residual):
    x, y, inv, w = _combine_case(dtype)
    out = synth.storage_to_f64(oracle.combine_topk(y, x, inv, w, residual))
    xf, yf = synth.storage_to_f64(x), synth.storage_to_f64(y)
    k, T = inv.shape
    for s in range(T):
        for c in range(x.shape[1]):
            if (inv[:, s] < 0).all():
                want = xf[s, c]
            else:
                acc = xf[s, c] if residual else 0.0
                for j in range(k):
                    if inv[j, s] >= 0:
                        acc += float(w[j, s]) * yf[inv[j, s], c]
                if dtype == synth.F32:
                    want = float(np.float32(acc))
                else:
                    want = float(torch.tensor(acc, dtype=torch.float64).to(torch.bfloat16))
            assert out[s, c] == want, (s, c)


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
@pytest.mark.parametrize("residual", [0, 1])
def test_combine_topk_k1_is_the_top1_combine(dtype, residual):
    x, y, inv, w = _combine_case(dtype, k=1, rows=30)
    a = oracle.combine_topk(y, x, inv, w, residual)
    b = oracle.combine(y, x, inv[0], w[0], residual)
    assert (a == b).all()


def test_combine_topk_passthrough_and_identity_experts():
    x, y, inv, w = _combine_case(synth.BF16)
    none = np.full_like(inv, -1)
    assert (oracle.combine_topk(y, x, none, w, 1) == x).all()
    assert (oracle.combine_topk(y, x, none, w, 0) == x).all()
    # every choice kept, every expert the identity, weights summing to one: out = x + x
    k, T = 3, x.shape[0]
    rows = np.ascontiguousarray(np.tile(x, (k, 1)))
    inv = np.arange(k * T, dtype=np.int32).reshape(k, T)
    w = np.random.default_rng(2).random((k, T))
    w = (w / w.sum(axis=0)).astype(np.float32)
    out = oracle.combine_topk(rows, x, inv, w, 1)
    assert np.array_equal(synth.storage_to_f64(out), 2 * synth.storage_to_f64(x))


# ------------------------------------------------------------------ whole layer
def _walk_layer(c, k, C_, cap_mult, renormalize, residual):
    """Assignment by assignment, first choices first: binary32 storage, float64 arithmetic."""
    x, wr, b = (synth.storage_to_f64(c[n]) for n in ("x", "w_router", "b_router"))
    w1, w2 = synth.storage_to_f64(c["w1"]), synth.storage_to_f64(c["w2"])
    T, E = x.shape[0], wr.shape[1]
    choice, weight = [], []
    for s in range(T):
        l = x[s] @ wr + b
        p = np.exp(l - l.max())
        p /= p.sum()
        ids = sorted(range(E), key=lambda e: (-l[e], e))[:k]
        ws = np.array([p[e] for e in ids])
        if renormalize:
            ws = ws / ws.sum()
        choice.append(ids)
        weight.append(ws.astype(np.float32).astype(np.float64))
    used = [0] * E
    out = np.array([x[s] if residual else np.zeros_like(x[s]) for s in range(T)])
    kept_any = [False] * T
    for j in range(k):
        for s in range(T):
            e = choice[s][j]
            if used[e] < cap_mult[e] * C_:
                used[e] += 1
                h = np.maximum(x[s] @ w1[e], 0).astype(np.float32).astype(np.float64)
                y = (h @ w2[e]).astype(np.float32).astype(np.float64)
                out[s] += weight[s][j] * y
                kept_any[s] = True
    for s in range(T):
        if not kept_any[s]:
            out[s] = x[s]
    return out.astype(np.float32), np.array(choice).T


@pytest.mark.parametrize("renormalize,residual,R", [(False, 1, 0), (True, 0, 0), (False, 1, 3)])
def test_layer_topk_against_assignment_walk(renormalize, residual, R):
    k, C_ = 3, 7
    c = synth.moe_layer_inputs(30, 8, 12, 6, synth.F32, 1.3, 33)
    got = oracle.layer_topk(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"], k, C_, R,
                            renormalize=renormalize, residual=residual)
    mult = got["plan"]["replicas"]
    if R == 0:
        assert (mult == 1).all()
    else:
        assert mult.sum() > len(mult)                        # the plan really granted replicas
    want, choice = _walk_layer(c, k, C_, mult, renormalize, residual)
    assert (got["route"]["idx"] == choice).all()
    assert (got["dispatch"]["inv"] < 0).any()                # capacity binds in this case
    assert np.allclose(got["out"], want, rtol=0, atol=2e-6)
