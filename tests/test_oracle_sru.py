"""Pins for the oracle's SRU predictor (CPU only): limiting cases and the unrolled closed
form of the equations in the paper's SRU subsection, plus state reset between sequences."""
import numpy as np
import torch

import oracle
import synth


def _one_layer(seed, B=2, L=9, n=6, n_out=5, n_in=None, bias=0.3):
    s = synth.sru_inputs(B, L, n_in or n, n, 1, n_out, synth.F32, seed, bias_std=bias, w_std=0.4)
    return s


def _run(s, **over):
    a = dict(s)
    a.update(over)
    return oracle.sru(a["emb"], a["w_cat"], a["b_f"], a["b_r"], a["w_head"], a["b_head"])


def _sig(v):
    return 1.0 / (1.0 + np.exp(-v))


def test_forget_gate_saturated_open_zeroes_the_state():
    s = _one_layer(1)
    n = 6
    out = _run(s, b_f=[np.full(n, 60.0, np.float32)])
    x = s["emb"].reshape(-1, n).astype(np.float64)
    r = _sig(x @ s["w_cat"][0][:, 2 * n:3 * n].astype(np.float64) + s["b_r"][0])
    assert np.allclose(out["h"], (1 - r) * x, rtol=1e-6, atol=1e-7)


def test_forget_gate_saturated_shut_removes_the_recurrence():
    s = _one_layer(2)
    n = 6
    out = _run(s, b_f=[np.full(n, -60.0, np.float32)])
    x = s["emb"].reshape(-1, n).astype(np.float64)
    w = s["w_cat"][0].astype(np.float64)
    r = _sig(x @ w[:, 2 * n:] + s["b_r"][0])
    assert np.allclose(out["h"], r * np.tanh(x @ w[:, :n]) + (1 - r) * x, rtol=1e-6, atol=1e-7)


def test_reset_gate_shut_is_identity_highway():
    s = _one_layer(3)
    out = _run(s, b_r=[np.full(6, -60.0, np.float32)])
    assert np.allclose(out["h"], s["emb"].reshape(-1, 6), rtol=1e-6, atol=1e-7)


def test_half_forget_constant_input_geometric_state():
    n, L = 4, 12
    s = _one_layer(4, B=1, L=L, n=n)
    emb = np.tile(s["emb"][:, :1, :], (1, L, 1)).copy()
    w = s["w_cat"][0].copy()
    w[:, n:2 * n] = 0.0                                   # W_f = 0, b_f = 0 -> f = 1/2
    out = _run(s, emb=emb, w_cat=[w], b_f=[np.zeros(n, np.float32)],
               b_r=[np.full(n, 60.0, np.float32)])       # r = 1 -> h = tanh(c)
    xp = emb[0, 0].astype(np.float64) @ w[:, :n].astype(np.float64)
    t = np.arange(L)[:, None]
    c = xp[None, :] * (1.0 - 2.0 ** -(t + 1.0))
    assert np.allclose(out["h"], np.tanh(c), rtol=1e-6, atol=1e-7)


def test_unrolled_closed_form_and_wide_input_highway():
    # n_in != n_hidden: the highway term is the fourth projection W_h x_t
    n, n_in, B, L = 5, 8, 2, 10
    s = _one_layer(5, B=B, L=L, n=n, n_in=n_in)
    out = _run(s)
    x = s["emb"].astype(np.float64)
    w = s["w_cat"][0].astype(np.float64)
    assert w.shape == (n_in, 4 * n)
    for b in range(B):
        u = x[b] @ w
        f = _sig(u[:, n:2 * n] + s["b_f"][0])
        r = _sig(u[:, 2 * n:3 * n] + s["b_r"][0])
        for t in range(L):
            c = np.zeros(n)
            for k in range(t + 1):
                c += np.prod(f[k + 1:t + 1], axis=0) * (1 - f[k]) * u[k, :n]
            h = r[t] * np.tanh(c) + (1 - r[t]) * u[t, 3 * n:]
            assert np.allclose(out["h"][b * L + t], h, rtol=1e-6, atol=1e-7)


def test_sequences_do_not_share_state():
    s = synth.sru_inputs(3, 7, 6, 6, 2, 4, synth.BF16, 6, bias_std=0.2, w_std=0.3)
    full = _run(s)
    for b in range(3):
        one = _run(s, emb=s["emb"][b:b + 1].copy())
        assert (full["h"][b * 7:(b + 1) * 7] == one["h"]).all()
        assert (full["pred"][b * 7:(b + 1) * 7] == one["pred"]).all()


def test_two_layers_compose_and_head_is_a_dense_product():
    s = synth.sru_inputs(2, 6, 10, 4, 2, 7, synth.BF16, 7, bias_std=0.2, w_std=0.3)
    full = _run(s)
    first = oracle.sru(s["emb"], s["w_cat"][:1], s["b_f"][:1], s["b_r"][:1], s["w_head"], None)
    second = oracle.sru(first["h"].reshape(2, 6, 4), s["w_cat"][1:], s["b_f"][1:], s["b_r"][1:],
                        s["w_head"], s["b_head"])
    assert (second["h"] == full["h"]).all()
    lg = torch.from_numpy(synth.storage_to_f64(full["h"])) @ \
        torch.from_numpy(synth.storage_to_f64(s["w_head"])) + torch.from_numpy(s["b_head"]).double()
    assert np.allclose(full["logits"], lg.numpy(), atol=1e-12)
    assert (full["pred"] == lg.numpy().argmax(1)).all()
    srt = np.sort(lg.numpy(), axis=1)
    assert np.allclose(full["margin"], srt[:, -1] - srt[:, -2], atol=1e-12)
