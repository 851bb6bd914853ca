"""Per-token brute force of the replicated MoE layer, in float64 numpy/Python loops.

TEST INFRASTRUCTURE ONLY, tiny inputs only (O(T^2) ranking, no sorting, no helper shared with
``moe_oracle.c``).  It follows the layer token by token: the token's own logits, its own
argmax and softmax probability, its rank among earlier tokens of the same expert, and the
chosen expert's FFN applied to that one row.  The replica plan is obtained by literally
walking the tokens as Algorithm 1 does (a token that finds every slot of its expert full asks
for one more physical replica), then applying the cap of the "Capacity capping" subsection.
"""
from __future__ import annotations

import numpy as np


def _f64(a):
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _store(v, like_dtype):
    """Round float64 values to the storage type (binary32, or bf16 returned as float64)."""
    v = np.asarray(v, np.float64)
    if like_dtype == np.float32:
        return v.astype(np.float32).astype(np.float64)
    out = np.empty_like(v)
    it = np.nditer(v, flags=["multi_index"])
    for a in it:
        a = float(a)
        if a == 0.0:
            out[it.multi_index] = a
            continue
        m, e = np.frexp(a)
        q = max(e - 8, -133)
        out[it.multi_index] = np.ldexp(np.rint(np.ldexp(a, -q)), q)
    return out


def wants_by_token_walk(ids, E, C):
    """Algorithm 1's inner loop with slots of C tokens: the first token of an expert loads it
    (one slot); a later token that finds all of the expert's slots full appends a replica."""
    slots = [0] * E
    held = [0] * E
    for e in ids:
        if slots[e] == 0:
            slots[e] = 1
            held[e] = 1
        elif held[e] < slots[e] * C:
            held[e] += 1
        else:
            slots[e] += 1
            held[e] += 1
    return [max(0, s - 1) for s in slots]


def plan(ids, E, R, C, policy=0):
    ids = [int(i) for i in ids]
    n = [ids.count(e) for e in range(E)]
    want = wants_by_token_walk(ids, E, C)
    r = [1] * E
    D = sum(want)
    if D <= R:
        return [1 + w for w in want]
    left = R
    if policy == 0:
        for e in range(E):
            r[e] += (R * want[e]) // D
        left = R - sum(x - 1 for x in r)
    else:
        while True:
            wanting = [e for e in range(E) if r[e] - 1 < want[e]]
            if not wanting or left // len(wanting) == 0:
                break
            q = left // len(wanting)
            for e in wanting:
                g = min(q, want[e] - (r[e] - 1))
                r[e] += g
                left -= g
    while left > 0:
        cand = [e for e in range(E) if r[e] - 1 < want[e]]
        if not cand:
            break
        # largest n_e / r_e as an exact fraction; lowest id on ties
        best = cand[0]
        for e in cand[1:]:
            if n[e] * r[best] > n[best] * r[e]:
                best = e
        r[best] += 1
        left -= 1
    return r


def layer(x, w_router, b_router, w1, w2, C, replicas, residual=0):
    """-> (idx, prob, kept flag, out) with one independent evaluation per token."""
    dt = x.dtype
    X, Wr, W1, W2 = _f64(x), _f64(w_router), _f64(w1), _f64(w2)
    T, d = X.shape
    E = Wr.shape[1]
    b = np.zeros(E) if b_router is None else np.asarray(b_router, np.float64)
    idx = np.empty(T, np.int64)
    prob = np.empty(T, np.float64)
    for s in range(T):
        l = np.array([sum(X[s, k] * Wr[k, e] for k in range(d)) + b[e] for e in range(E)])
        e = int(np.argmax(l))           # first maximum = lowest index
        idx[s] = e
        prob[s] = 1.0 / np.sum(np.exp(l - l[e]))
    prob32 = prob.astype(np.float32).astype(np.float64)
    out = np.empty((T, d), np.float64)
    kept = np.zeros(T, bool)
    for s in range(T):
        e = int(idx[s])
        j = sum(1 for t in range(s) if idx[t] == e)
        if j >= replicas[e] * C:
            out[s] = X[s]
            continue
        kept[s] = True
        h = np.maximum(X[s] @ W1[e], 0.0)
        h = _store(h, dt)
        y = _store(h @ W2[e], dt)
        out[s] = _store(prob32[s] * y + (X[s] if residual else 0.0), dt)
    return idx.astype(np.int32), prob32.astype(np.float32), kept, out
