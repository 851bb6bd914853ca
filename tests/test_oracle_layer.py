"""Pins for the oracle's router, expert FFN, combine and whole layer (CPU only).

Independent anchors: closed forms of the softmax router, a dense library product for the
single-expert special case (torch CPU float64 matmul), torch's own bfloat16 conversion for
the storage rounding, a separately written per-token brute force, and the paper's claim that
replication leaves the model's computation unchanged (Preliminaries; Conclusion).
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from oracle import brute_force as bf


def _tiny(dtype, seed, T=24, d=8, F=16, E=4, s=1.2):
    return synth.moe_layer_inputs(T, d, F, E, dtype, s, seed)


# ------------------------------------------------------------------ storage rounding
def test_bf16_storage_rounding_matches_torch():
    rng = np.random.default_rng(0)
    v = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-6, 6, 4000),
                        [0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.0e-39, 65280.0]])
    v32 = v.astype(np.float32)
    want = torch.from_numpy(v32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    # through the generator's bit trick
    assert (synth.bf16_bits(v32) == want).all()
    # through the oracle: combine with prob = 1 and residual = 0 stores y rounded once
    y = v32.reshape(-1, 1)
    yb = synth.bf16_bits(y)
    out = oracle.combine(yb, yb, np.arange(y.shape[0], dtype=np.int32),
                         np.ones(y.shape[0], np.float32))
    assert (out == yb).all()
    # and a product that needs rounding: prob * y, checked against torch in float64 -> bf16
    p = rng.random(y.shape[0]).astype(np.float32)
    out = oracle.combine(yb, yb, np.arange(y.shape[0], dtype=np.int32), p)
    exact = p.astype(np.float64)[:, None] * synth.storage_to_f64(yb)
    ref = torch.from_numpy(exact).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (out == ref).all()


# ------------------------------------------------------------------ router
def test_route_equal_logits_lowest_index_and_uniform_prob():
    x = np.ones((5, 6), np.float32)
    w = np.zeros((6, 7), np.float32)
    r = oracle.route(x, w, None)
    assert (r["idx"] == 0).all()
    assert np.allclose(r["prob"], 1.0 / 7.0, rtol=1e-7)
    assert (r["margin"] == 0).all()


def test_route_one_hot_router_known_argmax_and_softmax():
    rng = np.random.default_rng(1)
    T, d, E = 40, 10, 6
    x = rng.standard_normal((T, d)).astype(np.float32)
    w = np.zeros((d, E), np.float32)
    cols = [3, 7, 1, 0, 9, 4]
    for e, k in enumerate(cols):
        w[k, e] = 2.0
    b = rng.standard_normal(E).astype(np.float32)
    r = oracle.route(x, w, b)
    logits = 2.0 * x[:, cols].astype(np.float64) + b.astype(np.float64)
    assert np.allclose(r["logits"], logits, rtol=0, atol=1e-12)
    assert (r["idx"] == np.argmax(logits, axis=1)).all()
    sm = torch.softmax(torch.from_numpy(logits), dim=1).numpy()
    assert np.allclose(r["prob"], sm.max(axis=1), rtol=1e-6)
    srt = np.sort(logits, axis=1)
    assert np.allclose(r["margin"], srt[:, -1] - srt[:, -2], atol=1e-12)
    assert (r["idx2"] == np.argsort(logits, axis=1)[:, -2]).all()


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_route_matches_library_matmul(dtype):
    c = _tiny(dtype, 7, T=33, d=20, E=9)
    r = oracle.route(c["x"], c["w_router"], c["b_router"])
    ref = torch.from_numpy(synth.storage_to_f64(c["x"])) @ \
        torch.from_numpy(synth.storage_to_f64(c["w_router"])) + torch.from_numpy(c["b_router"]).double()
    assert np.allclose(r["logits"], ref.numpy(), rtol=0, atol=1e-12)


def test_route_transposed_operand_would_fail():
    # a square, asymmetric router: x @ W and x @ W^T disagree, the oracle follows x @ W
    rng = np.random.default_rng(2)
    x = rng.standard_normal((9, 5)).astype(np.float32)
    w = rng.standard_normal((5, 5)).astype(np.float32)
    r = oracle.route(x, w, None)
    assert np.allclose(r["logits"], x.astype(np.float64) @ w.astype(np.float64), atol=1e-12)
    assert not np.allclose(r["logits"], x.astype(np.float64) @ w.T.astype(np.float64), atol=1e-3)


# ------------------------------------------------------------------ FFN
@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_single_expert_reduces_to_dense_library_product(dtype):
    c = _tiny(dtype, 3, T=19, d=12, F=28, E=1)
    T = c["T"]
    so = np.array([0, T], np.int32)
    se = np.array([0], np.int32)
    y, h = oracle.ffn(c["x"], c["w1"], c["w2"], so, se, 1, want_h=True)
    X = torch.from_numpy(synth.storage_to_f64(c["x"]))
    W1 = torch.from_numpy(synth.storage_to_f64(c["w1"][0]))
    W2 = torch.from_numpy(synth.storage_to_f64(c["w2"][0]))
    hd = torch.relu(X @ W1)
    if dtype == synth.BF16:
        href = hd.to(torch.bfloat16)
        assert (h == href.view(torch.int16).numpy().view(np.uint16)).mean() > 0.995
        yref = (synth.storage_to_f64(h) @ W2.numpy())
        got = synth.storage_to_f64(y)
        assert np.abs(got - yref).max() <= 2.0 ** -8 * np.abs(yref).max()
        dense = (hd @ W2).numpy()
        assert np.abs(got - dense).max() <= 2e-2 * np.abs(dense).max()
    else:
        assert np.allclose(h, hd.numpy(), rtol=1e-6, atol=1e-9)
        assert np.allclose(y, (hd @ W2).numpy(), rtol=1e-5, atol=1e-8)


def test_ffn_uses_the_slot_owner_weights_and_row_subset():
    c = _tiny(synth.F32, 4, T=12, d=6, F=10, E=3)
    so = np.array([0, 4, 4, 9, 12], np.int32)       # slot 1 empty
    se = np.array([2, 0, 0, 1], np.int32)
    y = oracle.ffn(c["x"], c["w1"], c["w2"], so, se, 4)
    X = c["x"].astype(np.float64)
    for row in range(12):
        e = [2, 2, 2, 2, 0, 0, 0, 0, 0, 1, 1, 1][row]
        h = np.maximum(X[row] @ c["w1"][e].astype(np.float64), 0).astype(np.float32).astype(np.float64)
        assert np.allclose(y[row], h @ c["w2"][e].astype(np.float64), rtol=1e-5, atol=1e-9)
    sub = oracle.ffn(c["x"], c["w1"], c["w2"], so, se, 4, rows=[10, 1])
    assert (sub[[10, 1]] == y[[10, 1]]).all() and (np.delete(sub, [10, 1], 0) == 0).all()


# ------------------------------------------------------------------ combine
def test_combine_passthrough_bits_and_unpermute():
    rng = np.random.default_rng(5)
    T, d = 30, 7
    for dtype in (synth.F32, synth.BF16):
        x = synth.f32_to_storage(rng.standard_normal((T, d)), dtype)
        y = synth.f32_to_storage(rng.standard_normal((T, d)), dtype)
        perm = rng.permutation(T)[:20]
        inv = np.full(T, -1, np.int32)
        inv[perm] = np.arange(20)
        out = oracle.combine(y, x, inv, np.ones(T, np.float32), 0)
        assert (out[inv < 0] == x[inv < 0]).all()                 # dropped rows: bit copies
        assert (out[perm] == y[:20]).all()                        # prob 1: pure un-permute
        p = rng.random(T).astype(np.float32)
        out = oracle.combine(y, x, inv, p, 1)
        ref = synth.storage_to_f64(x)[perm] + p[perm].astype(np.float64)[:, None] * synth.storage_to_f64(y)[:20]
        got = synth.storage_to_f64(out)[perm]
        tol = 1e-6 if dtype == synth.F32 else 2.0 ** -8
        assert np.abs(got - ref).max() <= tol * np.abs(ref).max()
        assert (out[inv < 0] == x[inv < 0]).all()


# ------------------------------------------------------------------ whole layer
@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
@pytest.mark.parametrize("residual", [0, 1])
def test_layer_matches_per_token_brute_force(dtype, residual):
    for seed, C, R in [(21, 3, 0), (22, 3, 3), (23, 5, 2), (24, 100, 0), (25, 1, 6)]:
        c = _tiny(dtype, seed)
        L = oracle.layer(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"], C, R,
                         residual=residual)
        idx, prob, kept, out = bf.layer(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"],
                                        C, list(L["plan"]["replicas"]), residual)
        assert (L["route"]["idx"] == idx).all()
        assert np.allclose(L["route"]["prob"], prob, rtol=1e-6)
        assert ((L["dispatch"]["inv"] >= 0) == kept).all()
        assert list(L["plan"]["replicas"]) == bf.plan(idx, c["E"], R, C, 0)
        got = synth.storage_to_f64(L["out"])
        if dtype == synth.F32:
            assert np.allclose(got, out, rtol=1e-6, atol=1e-9)
        else:
            # same roundings on both sides; a different summation order inside the library
            # matmul can move a value across one bf16 rounding boundary
            assert np.abs(got - out).max() <= 2.0 ** -7 * np.abs(out).max()
            assert (got == out).mean() > 0.98
        assert (L["out"][~kept] == c["x"][~kept]).all()


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_replication_leaves_outputs_unchanged(dtype):
    """With room for every token (C >= T) any replica plan gives bit-identical outputs; with
    drops, a plan equals a run without slots under the per-expert capacity vector r_e*C."""
    c = _tiny(dtype, 31, T=60, E=5)
    big = oracle.layer(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"], 60, 0)
    ids = big["route"]["idx"]
    for R, C in [(0, 60), (7, 60)]:
        forged = np.arange(60, dtype=np.int32) % 5       # any plan input: outputs must not move
        L = oracle.layer(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"], C, R, plan_ids=forged)
        assert (L["out"] == big["out"]).all()
    # with drops: explicit replicas vs one slot per expert with capacity r_e*C
    C, R = 4, 6
    L = oracle.layer(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"], C, R)
    r = L["plan"]["replicas"]
    n = np.bincount(ids, minlength=5)
    keep_cap = np.minimum(n, r * C)
    off = np.concatenate([[0], np.cumsum(keep_cap)]).astype(np.int32)
    y1 = oracle.ffn(L["dispatch"]["x_perm"], c["w1"], c["w2"], off, np.arange(5, dtype=np.int32), 5)
    assert (y1 == L["y_perm"]).all()
    assert (L["dispatch"]["expert_offset"] == off).all()
    assert int((L["dispatch"]["inv"] < 0).sum()) == 60 - keep_cap.sum()


def test_config1_has_two_or_three_overloaded_experts_and_no_drops():
    c = synth.config_inputs(1)
    L = oracle.layer(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"], c["C"], c["R"])
    n = L["plan"]["counts"]
    assert 2 <= int((n > c["C"]).sum()) <= 3
    assert n.sum() == c["T"]
    assert (L["plan"]["replicas"] - 1).sum() <= c["R"]


def test_token_count_conservation_config1():
    c = synth.config_inputs(1)
    for R in (0, 2, 4):
        L = oracle.layer(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"], c["C"], R)
        K = int(L["dispatch"]["kept"].sum())
        dropped = L["dispatch"]["inv"] < 0
        assert K + int(dropped.sum()) == c["T"]
        assert (L["out"][dropped] == c["x"][dropped]).all()
