"""Pins for the oracle's sparsemax attention, independent of the oracle's own
formula: closed forms, invariants, a bisection solve of the projection, and limiting cases of the
attention in which the result is known without computing it."""
import numpy as np
import pytest

import oracle
import synth
from oracle.sparse_attention import attend, head, sparsemax


def _simplex_projection_by_bisection(z):
    """Independent route to the same object: the projection onto the simplex is max(z - tau, 0) with
    the unique tau at which the entries sum to one; bisect on tau."""
    lo, hi = z.min() - 1.0, z.max()
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if np.maximum(z - mid, 0.0).sum() > 1.0:
            lo = mid
        else:
            hi = mid
    return np.maximum(z - 0.5 * (lo + hi), 0.0)


@pytest.mark.parametrize("seed", range(6))
def test_sparsemax_is_the_simplex_projection(seed):
    rng = np.random.default_rng(seed)
    z = rng.normal(0, [0.1, 1.0, 5.0][seed % 3], size=[3, 17, 512][seed % 3])
    p = sparsemax(z)
    assert p.min() >= 0 and abs(p.sum() - 1.0) < 1e-12
    assert np.abs(p - _simplex_projection_by_bisection(z)).max() < 1e-10
    # any other point of the simplex is farther from z
    for _ in range(20):
        q = rng.dirichlet(np.ones(z.size))
        assert np.sum((q - z) ** 2) >= np.sum((p - z) ** 2) - 1e-12
    # invariance under a shift, equivariance under a permutation
    assert np.abs(sparsemax(z + 3.7) - p).max() < 1e-12
    perm = rng.permutation(z.size)
    assert np.abs(sparsemax(z[perm]) - p[perm]).max() < 1e-12


def test_sparsemax_closed_forms():
    # two entries: p1 = clip((1 + z1 - z2) / 2, 0, 1)
    for z1, z2 in [(0.0, 0.0), (0.3, -0.2), (2.0, 0.0), (-1.0, 0.5), (0.5, 1.5)]:
        p = sparsemax(np.array([z1, z2]))
        want = min(1.0, max(0.0, (1.0 + z1 - z2) / 2.0))
        assert abs(p[0] - want) < 1e-15 and abs(p[1] - (1 - want)) < 1e-15
    # equal entries -> uniform; one entry ahead by >= 1 -> one-hot with exact zeros elsewhere
    assert np.allclose(sparsemax(np.full(7, 0.3)), 1 / 7)
    p = sparsemax(np.array([0.125, 1.25, 0.25, -3.0]))
    assert p[1] == 1.0 and (np.delete(p, 1) == 0.0).all()
    # a worked three-entry case: z = (1, 0.5, -1): support {1, 2}, tau = 0.25
    assert np.allclose(sparsemax(np.array([1.0, 0.5, -1.0])), [0.75, 0.25, 0.0])
    # sparse: zeros are exact, and a softmax would give every entry weight
    z = np.linspace(-2, 2, 50)
    p = sparsemax(z)
    assert (p == 0).sum() >= 40 and abs(p.sum() - 1) < 1e-12


def test_attention_limiting_cases():
    f64 = lambda a: a.astype(np.float64)
    ident = lambda a: a
    B, L, n = 2, 6, 8
    # (a) every state of a sequence equal: uniform attention, context = the state itself, z = 2 h
    h = np.repeat(np.arange(1, B + 1, dtype=np.float64)[:, None, None], L, 1) * np.ones((B, L, n))
    z = attend(h.reshape(B * L, n), B, L, f64, ident)
    assert np.allclose(z, 2 * h.reshape(B * L, n))
    # (b) mutually orthogonal states of large norm: each position attends to itself only
    h = np.zeros((B, L, n))
    for b in range(B):
        for t in range(L):
            h[b, t, t] = 10.0 * (1 + b)
    z = attend(h.reshape(B * L, n), B, L, f64, ident)
    assert np.array_equal(z, 2 * h.reshape(B * L, n))
    # (c) no attention across sequences: changing sequence 1 leaves sequence 0's rows alone
    rng = np.random.default_rng(0)
    h = rng.normal(size=(B, L, n))
    z0 = attend(h.reshape(B * L, n), B, L, f64, ident)
    h2 = h.copy()
    h2[1] = rng.normal(size=(L, n))
    z1 = attend(h2.reshape(B * L, n), B, L, f64, ident)
    assert np.array_equal(z0[:L], z1[:L]) and not np.array_equal(z0[L:], z1[L:])
    # (d) the context is a convex combination of the sequence's states: per coordinate it lies between their extremes
    c = z0 - h.reshape(B * L, n)
    for b in range(B):
        blk = h[b]
        assert (c[b * L:(b + 1) * L] <= blk.max(0) + 1e-12).all() and (c[b * L:(b + 1) * L] >= blk.min(0) - 1e-12).all()


def test_head_and_full_predictor_consistency():
    s = synth.sru_inputs(2, 24, 64, 64, 2, 16, synth.BF16, 12, bias_std=0.2, w_std=0.1)
    full = oracle.sru_attention(s["emb"], s["w_cat"], s["b_f"], s["b_r"], s["w_head"], s["b_head"])
    base = oracle.sru(s["emb"], s["w_cat"], s["b_f"], s["b_r"], s["w_head"], s["b_head"])
    assert np.array_equal(full["h"], base["h"])
    # z is stored in bf16 and differs from h by a convex combination of the states
    hf, zf = synth.storage_to_f64(full["h"]), synth.storage_to_f64(full["z"])
    c = zf - hf
    for b in range(2):
        blk = hf[b * 24:(b + 1) * 24]
        tol = 2.0 ** -7 * (np.abs(blk).max() * 2)
        assert (c[b * 24:(b + 1) * 24] <= blk.max(0) + tol).all() and (c[b * 24:(b + 1) * 24] >= blk.min(0) - tol).all()
    # the head: numpy matmul re-derivation of argmax / margin on the stored z
    lg = zf @ synth.storage_to_f64(s["w_head"]) + s["b_head"].astype(np.float64)
    assert np.array_equal(full["pred"], lg.argmax(1))
    top2 = np.sort(lg, 1)[:, -2:]
    assert np.allclose(full["margin"], top2[:, 1] - top2[:, 0])
    # one-rounding storage: every z is within half a bf16 ulp (spacing 2^-7 of the binade) of h + c recomputed here
    z_exact = np.empty_like(hf)
    for b in range(2):
        hb = hf[b * 24:(b + 1) * 24]
        sc = hb @ hb.T / 8.0
        for t in range(24):
            z_exact[b * 24 + t] = hb[t] + sparsemax(sc[t]) @ hb
    assert (np.abs(zf - z_exact) <= 2.0 ** -8 * np.abs(z_exact) + 1e-30).all()
