"""CPU oracle of the replicated top-1 MoE layer.  TEST INFRASTRUCTURE ONLY.

``moe_oracle.c`` (plain C, double arithmetic) holds the definitions; this module compiles
it with gcc and marshals numpy arrays into it.  ``brute_force.py`` is a second, per-token
evaluation in Python used to cross-check the C code on tiny inputs.  Nothing in the product
package may import this package; only tests, the smoke check and the bench's CPU-baseline
leg do.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc -O2 -fopenmp) next to its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c11", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        for name in ("orc_route", "orc_sru", "orc_plan", "orc_dispatch", "orc_ffn",
                     "orc_combine", "orc_num_threads", "orc_set_num_threads"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def num_threads() -> int:
    return lib().orc_num_threads()


def set_num_threads(n: int) -> int:
    """Threads for the parallel loops from now on (timing only); returns the number in force."""
    return lib().orc_set_num_threads(int(n))


def _st(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError(f"storage must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _p(a):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def _chk(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid arguments")


def _to_storage(a, st):
    """float64 -> storage in one rounding (nearest, ties to even)."""
    if st == 0:
        return a.astype(np.float32)
    m, e = np.frexp(a)                                  # bf16: 8 significant bits
    r = np.ldexp(np.rint(np.ldexp(m, 8)), e - 8)        # exactly representable in binary32 and in bf16
    return (r.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)


def route(x, w_router, b_router=None):
    """-> dict(idx int32[T], prob f32[T], logits f64[T,E], idx2 int32[T], margin f64[T])."""
    T, d = x.shape
    E = w_router.shape[1]
    st = _st(x)
    assert _st(w_router) == st and w_router.shape[0] == d
    idx = np.empty(T, np.int32)
    prob = np.empty(T, np.float32)
    logits = np.empty((T, E), np.float64)
    idx2 = np.empty(T, np.int32)
    margin = np.empty(T, np.float64)
    b = None if b_router is None else np.ascontiguousarray(b_router, np.float32)
    _chk(lib().orc_route(_p(x), _p(w_router), _p(b), T, d, E, st, _p(idx), _p(prob),
                         _p(logits), _p(idx2), _p(margin)), "route")
    return dict(idx=idx, prob=prob, logits=logits, idx2=idx2, margin=margin)


def sru(emb, w_cat, b_f, b_r, w_head, b_head=None):
    """emb [B,L,n_in]; w_cat list per layer.  -> dict(pred, logits, idx2, margin, h)."""
    B, L, n_in = emb.shape
    st = _st(emb)
    n_layers = len(w_cat)
    n_h, n_out = w_head.shape
    T = B * L
    PT = C.c_void_p * n_layers
    wc = PT(*[w.ctypes.data for w in w_cat])
    bfs = [None if b is None else np.ascontiguousarray(b, np.float32) for b in (b_f or [None] * n_layers)]
    brs = [None if b is None else np.ascontiguousarray(b, np.float32) for b in (b_r or [None] * n_layers)]
    if any(b is None for b in bfs + brs):
        bfs = [np.zeros(n_h, np.float32) if b is None else b for b in bfs]
        brs = [np.zeros(n_h, np.float32) if b is None else b for b in brs]
    bfp = PT(*[b.ctypes.data for b in bfs])
    brp = PT(*[b.ctypes.data for b in brs])
    bh = None if b_head is None else np.ascontiguousarray(b_head, np.float32)
    pred = np.empty(T, np.int32)
    logits = np.empty((T, n_out), np.float64)
    idx2 = np.empty(T, np.int32)
    margin = np.empty(T, np.float64)
    h = np.empty((T, n_h), emb.dtype)
    for l, w in enumerate(w_cat):
        nin = n_in if l == 0 else n_h
        k = 3 if nin == n_h else 4
        assert w.shape == (nin, k * n_h) and _st(w) == st and w.flags["C_CONTIGUOUS"]
    _chk(lib().orc_sru(_p(emb), B, L, n_layers, n_in, n_h, n_out, wc, bfp, brp, _p(w_head),
                       _p(bh), st, _p(pred), _p(logits), _p(idx2), _p(margin), _p(h)), "sru")
    return dict(pred=pred, logits=logits, idx2=idx2, margin=margin, h=h)


def sru_attention(emb, w_cat, b_f, b_r, w_head, b_head=None):
    """The SRU predictor with sparsemax attention over its last layer's states
    (``oracle/sparse_attention.py`` states the reading).  -> dict(pred, logits, idx2, margin, h, z)."""
    import synth
    from . import sparse_attention as sa
    base = sru(emb, w_cat, b_f, b_r, w_head, b_head)
    B, L, _ = emb.shape
    st = _st(emb)

    def to_storage(a):
        return _to_storage(a, st)

    z = sa.attend(base["h"], B, L, synth.storage_to_f64, to_storage)
    out = sa.head(z, w_head, b_head, synth.storage_to_f64)
    out["h"], out["z"] = base["h"], z
    return out


def plan(idx, E, R, C_, policy=0):
    """-> dict(counts[E], replicas[E], slot_base[E+1], slot_expert[E+R], n_slots)."""
    idx = np.ascontiguousarray(idx, np.int32)
    counts = np.empty(E, np.int32)
    replicas = np.empty(E, np.int32)
    slot_base = np.empty(E + 1, np.int32)
    slot_expert = np.full(E + R, -1, np.int32)
    n_slots = np.zeros(1, np.int32)
    _chk(lib().orc_plan(_p(idx), idx.shape[0], E, R, C_, policy, _p(counts), _p(replicas),
                        _p(slot_base), _p(slot_expert), _p(n_slots)), "plan")
    return dict(counts=counts, replicas=replicas, slot_base=slot_base, slot_expert=slot_expert,
                n_slots=int(n_slots[0]))


def dispatch(x, idx, replicas, E, C_, max_slots):
    """-> dict(counts, kept, expert_offset, slot_offset, perm, inv, x_perm)."""
    T, d = x.shape
    idx = np.ascontiguousarray(idx, np.int32)
    rep = None if replicas is None else np.ascontiguousarray(replicas, np.int32)
    counts = np.empty(E, np.int32)
    kept = np.empty(E, np.int32)
    expert_offset = np.empty(E + 1, np.int32)
    slot_offset = np.empty(max_slots + 1, np.int32)
    perm = np.empty(T, np.int32)
    inv = np.empty(T, np.int32)
    x_perm = np.zeros_like(x)
    _chk(lib().orc_dispatch(_p(x), _p(idx), _p(rep), T, d, E, C_, max_slots, _st(x), _p(counts),
                            _p(kept), _p(expert_offset), _p(slot_offset), _p(perm), _p(inv),
                            _p(x_perm)), "dispatch")
    return dict(counts=counts, kept=kept, expert_offset=expert_offset, slot_offset=slot_offset,
                perm=perm, inv=inv, x_perm=x_perm)


def ffn(x_perm, w1, w2, slot_offset, slot_expert, n_slots, rows=None, want_h=False):
    """-> y_perm (and h when want_h).  rows: optional int32 list of permuted rows to evaluate."""
    d = x_perm.shape[1]
    F = w1.shape[2]
    st = _st(x_perm)
    assert _st(w1) == st and _st(w2) == st and w1.shape[1] == d and w2.shape[1:] == (F, d)
    y = np.zeros_like(x_perm)
    h = np.zeros((x_perm.shape[0], F), x_perm.dtype) if want_h else None
    so = np.ascontiguousarray(slot_offset, np.int32)
    se = np.ascontiguousarray(slot_expert, np.int32)
    r = None if rows is None else np.ascontiguousarray(rows, np.int32)
    _chk(lib().orc_ffn(_p(x_perm), _p(w1), _p(w2), _p(so), _p(se), int(n_slots), d, F, st, _p(r),
                       0 if r is None else r.shape[0], _p(y), _p(h)), "ffn")
    return (y, h) if want_h else y


def combine(y_perm, x, inv, prob, residual=0):
    T, d = x.shape
    out = np.empty_like(x)
    inv = np.ascontiguousarray(inv, np.int32)
    prob = np.ascontiguousarray(prob, np.float32)
    _chk(lib().orc_combine(_p(y_perm), _p(x), _p(inv), _p(prob), T, d, _st(x), int(residual),
                           _p(out)), "combine")
    return out


def layer(x, w_router, b_router, w1, w2, C_, R, policy=0, plan_ids=None, residual=0,
          idx=None, prob=None, rows=None):
    """Whole layer: route -> plan (from plan_ids, default the router's own ids) -> dispatch
    -> expert FFN -> combine.  ``idx``/``prob`` may be supplied to teacher-force the integer
    routing decision.  -> dict with every intermediate."""
    E = w_router.shape[1]
    rt = route(x, w_router, b_router)
    if idx is not None:
        rt = dict(rt, idx=np.ascontiguousarray(idx, np.int32))
    if prob is not None:
        rt = dict(rt, prob=np.ascontiguousarray(prob, np.float32))
    pl = plan(rt["idx"] if plan_ids is None else plan_ids, E, R, C_, policy)
    dp = dispatch(x, rt["idx"], pl["replicas"], E, C_, E + R)
    y = ffn(dp["x_perm"], w1, w2, dp["slot_offset"], pl["slot_expert"], pl["n_slots"], rows=rows)
    out = combine(y, x, dp["inv"], rt["prob"], residual)
    return dict(route=rt, plan=pl, dispatch=dp, y_perm=y, out=out)


def route_topk(x, w_router, b_router, k, renormalize=False):
    """Top-k router (``oracle/topk.py`` states the reading): the logits of ``route`` and the k
    largest of them per token.  -> dict(idx int32 [k,T], weight f32 [k,T], gap f64 [T], logits)."""
    from . import topk
    rt = route(x, w_router, b_router)
    sel = topk.select(rt["logits"], k, renormalize)
    return dict(idx=sel["idx"], weight=sel["weight"].astype(np.float32), gap=sel["gap"],
                logits=rt["logits"])


def combine_topk(y_perm, x, inv, weight, residual=0):
    """inv int32 [k,T], weight f32 [k,T] -> out in the storage type of x (one rounding)."""
    import synth
    from . import topk
    st = _st(x)
    inv = np.ascontiguousarray(inv, np.int32)
    out, passthrough = topk.combine(synth.storage_to_f64(y_perm), synth.storage_to_f64(x), inv,
                                    np.asarray(weight, np.float32).astype(np.float64), bool(residual))
    res = _to_storage(out, st)
    res[passthrough] = x[passthrough]
    return res


def layer_topk(x, w_router, b_router, w1, w2, k, C_, R, policy=0, renormalize=False, residual=0,
               idx=None, weight=None, rows=None):
    """Whole top-k layer: route_topk -> plan / dispatch / expert FFN over the k*T assignments
    (choice-major) -> combine_topk.  ``idx``/``weight`` [k,T] may be supplied to teacher-force the
    routing decision.  -> dict with every intermediate."""
    from . import topk
    E = w_router.shape[1]
    T = x.shape[0]
    rt = route_topk(x, w_router, b_router, k, renormalize)
    if idx is not None:
        rt = dict(rt, idx=np.ascontiguousarray(idx, np.int32).reshape(k, T))
    if weight is not None:
        rt = dict(rt, weight=np.ascontiguousarray(weight, np.float32).reshape(k, T))
    ids = rt["idx"].reshape(-1)
    pl = plan(ids, E, R, C_, policy)
    dp = dispatch(topk.assignment_rows(x, k), ids, pl["replicas"], E, C_, E + R)
    y = ffn(dp["x_perm"], w1, w2, dp["slot_offset"], pl["slot_expert"], pl["n_slots"], rows=rows)
    out = combine_topk(y, x, dp["inv"].reshape(k, T), rt["weight"], residual)
    return dict(route=rt, plan=pl, dispatch=dp, y_perm=y, out=out)
