"""Top-k routing on the replicated MoE layer (the experimental setup runs one task with top-3
routing instead of top-1).  TEST INFRASTRUCTURE ONLY, float64 numpy.

The paper names the setting and nothing more, so this module fixes a reading, the usual one for a
softmax-gated layer, and the HIP path is held to it:

* gate: p = softmax(logits) over all E experts (the router of the top-1 layer, unchanged);
* choice j = 0..k-1 of token s is the expert with the j-th largest logit, the lower id first
  among equal logits (k = 1 is the top-1 router);
* the weight of choice j is p[e_j], or p[e_j] / (p[e_0] + .. + p[e_{k-1}]) with ``renormalize``;
* an assignment is the pair (choice j, token s), numbered a = j*T + s: all first choices come
  before all second choices, so under the capacity limit a token's first choice is served before
  anybody's second choice.  Planning, dispatch and the expert FFN treat the k*T assignments
  exactly like k*T tokens of a top-1 layer whose row a is the row of token a mod T;
* out[s] = x[s] (with the residual option) + sum over the kept choices j of weight_j * y_j, where
  y_j is the expert output of assignment (j, s); choices over capacity drop out of the sum; a token
  with no kept choice passes through bit for bit, as in the top-1 layer.
"""
from __future__ import annotations

import numpy as np


def select(logits: np.ndarray, k: int, renormalize: bool = False) -> dict:
    """logits float64 [T,E] -> dict(idx int32 [k,T], weight float64 [k,T], gap float64 [T]).

    ``gap`` is the smallest difference between consecutive logits among the k+1 largest of a token
    (inf when E == k and k == 1): where it is large the ids and their order are beyond doubt."""
    logits = np.asarray(logits, np.float64)
    T, E = logits.shape
    assert 1 <= k <= E
    z = np.exp(logits - logits.max(axis=1, keepdims=True))
    p = z / z.sum(axis=1, keepdims=True)
    left = logits.copy()
    idx = np.empty((k, T), np.int32)
    top = np.empty((k + 1, T), np.float64)
    rows = np.arange(T)
    for j in range(k):
        e = left.argmax(axis=1)                 # the first maximum: lowest id among equals
        idx[j] = e
        top[j] = left[rows, e]
        left[rows, e] = -np.inf
    top[k] = left.max(axis=1) if E > k else -np.inf
    weight = p[rows[None, :], idx]
    if renormalize:
        weight = weight / weight.sum(axis=0, keepdims=True)
    gap = (top[:-1] - top[1:]).min(axis=0)
    return dict(idx=idx, weight=weight, gap=gap)


def assignment_rows(x: np.ndarray, k: int) -> np.ndarray:
    """The k*T rows the top-1 machinery sees: row j*T + s is the row of token s."""
    return np.ascontiguousarray(np.tile(x, (k, 1)))


def combine(y_perm_f64: np.ndarray, x_f64: np.ndarray, inv: np.ndarray, weight: np.ndarray,
            residual: bool) -> tuple:
    """y_perm_f64 [rows,d], x_f64 [T,d] (values of the stored tensors), inv int [k,T] (row of
    assignment (j,s) or -1), weight [k,T] -> (out float64 [T,d] before rounding to storage,
    passthrough bool [T]: tokens whose output is x[s] itself)."""
    k, T = inv.shape
    out = x_f64.copy() if residual else np.zeros_like(x_f64)
    any_kept = np.zeros(T, bool)
    for j in range(k):
        kept = inv[j] >= 0
        any_kept |= kept
        out[kept] += np.asarray(weight[j], np.float64)[kept, None] * y_perm_f64[inv[j][kept]]
    out[~any_kept] = x_f64[~any_kept]
    return out, ~any_kept
