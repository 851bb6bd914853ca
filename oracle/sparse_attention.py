"""Sparsemax attention over the SRU states and the predictor head on top of it (oracle side).

TEST INFRASTRUCTURE ONLY -- plain numpy in float64, no blocking, nothing shared with the HIP path.

The paper says the predictor is an SRU "with sparse attention" (Methodology) and that sparsemax
turns the attention weights into a sparse distribution that gives less relevant tokens exactly
zero weight (last paragraph of the SRU subsection); it prints no equations for it.  The reading
taken here (stated with its alternatives in the design notes):

  * one parameter-free self-attention over the states h_t of the LAST SRU layer, inside each of the
    B sequences (no attention across sequences, all L positions visible to every position);
  * scores s[t, j] = <h_t, h_j> / sqrt(n_hidden), on the states as stored (dtype-rounded);
  * a[t, :] = sparsemax(s[t, :]);
  * context c_t = sum_j a[t, j] h_j;  features z_t = h_t + c_t, rounded to the storage dtype;
  * logits = z_t W_head + b_head, prediction = argmax (lowest index on ties).

sparsemax(z) is the Euclidean projection of z onto the probability simplex (Martins & Astudillo,
2016): with z sorted in decreasing order, k* = max{k : 1 + k z_(k) > sum_{i<=k} z_(i)},
tau = (sum_{i<=k*} z_(i) - 1) / k*, p_i = max(z_i - tau, 0).
"""
from __future__ import annotations

import numpy as np


def sparsemax(z: np.ndarray) -> np.ndarray:
    """Sparsemax of a 1-D array, by the sorting definition.  float64 in and out."""
    z = np.asarray(z, np.float64)
    if z.ndim != 1 or z.size == 0:
        raise ValueError("sparsemax takes a non-empty 1-D array")
    zs = np.sort(z)[::-1]
    cs = np.cumsum(zs)
    k = np.arange(1, z.size + 1, dtype=np.float64)
    in_support = 1.0 + k * zs > cs
    k_star = int(np.nonzero(in_support)[0].max()) + 1
    tau = (cs[k_star - 1] - 1.0) / k_star
    return np.maximum(z - tau, 0.0)


def attend(h: np.ndarray, B: int, L: int, to_f64, to_storage) -> np.ndarray:
    """h: states of the last SRU layer as stored, [B*L, n].  Returns z (storage dtype), [B*L, n]."""
    T, n = h.shape
    if T != B * L:
        raise ValueError("h must have B*L rows")
    hf = to_f64(h)
    z = np.empty((T, n), np.float64)
    scale = 1.0 / np.sqrt(float(n))
    for b in range(B):
        hb = hf[b * L:(b + 1) * L]
        s = (hb @ hb.T) * scale
        for t in range(L):
            a = sparsemax(s[t])
            z[b * L + t] = hb[t] + a @ hb
    return to_storage(z)


def head(z: np.ndarray, w_head: np.ndarray, b_head, to_f64) -> dict:
    """logits, argmax (lowest index on ties), runner-up and their gap."""
    lg = to_f64(z) @ to_f64(w_head)
    if b_head is not None:
        lg = lg + np.asarray(b_head, np.float64)[None, :]
    pred = np.argmax(lg, axis=1).astype(np.int32)
    masked = lg.copy()
    masked[np.arange(lg.shape[0]), pred] = -np.inf
    idx2 = np.argmax(masked, axis=1).astype(np.int32) if lg.shape[1] > 1 else pred.copy()
    margin = lg[np.arange(lg.shape[0]), pred] - (masked.max(axis=1) if lg.shape[1] > 1 else 0.0)
    return dict(pred=pred, logits=lg, idx2=idx2, margin=margin)
