"""ctypes binding of ``libmoe_mpmc.so``: the library's calls under the same names (the six steps
of the layer, weight packing, the fused plan + dispatch front end, the top-k variants) on torch
tensors, and three small classes that hold preallocated buffers and issue the calls in order.
Argument marshalling only -- every step of the path runs in the HIP kernels.  Torch is used for
device memory and the current stream, nothing else.  There is no CPU fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

MOE_F32, MOE_BF16 = 0, 1
LAYOUT_PLAIN, LAYOUT_PACKED = 0, 1
SCHEDULE_SLOTS, SCHEDULE_EXPERTS = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_mpmc.so")
_lib = None

EXPORTS = (
    "moe_last_error", "moe_version", "moe_build_id",
    "moe_route_workspace_bytes", "moe_route",
    "sru_predict_workspace_bytes", "sru_predict",
    "replica_plan_workspace_bytes", "replica_plan",
    "moe_dispatch_workspace_bytes", "moe_dispatch", "moe_dispatch_static",
    "moe_packed_weights_bytes", "moe_pack_weights",
    "moe_expert_ffn_workspace_bytes", "moe_expert_ffn", "moe_expert_ffn_timed",
    "moe_combine",
    "moe_route_topk", "moe_dispatch_topk", "moe_expert_ffn_rows", "moe_combine_topk",
    "moe_plan_dispatch_workspace_bytes", "moe_plan_dispatch",
    "moe_measure_sink_bytes", "moe_measure_stream_read", "moe_measure_mfma_bf16_flops", "moe_measure_mfma_bf16",
)


class MoeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"[{code}] {msg}")
        self.code = code


class SruWeightsC(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("n_in", C.c_int), ("n_hidden", C.c_int), ("n_out", C.c_int),
                ("w_layout", C.c_int), ("w_cat", C.POINTER(C.c_void_p)), ("b_f", C.POINTER(C.c_void_p)),
                ("b_r", C.POINTER(C.c_void_p)), ("w_head", C.c_void_p), ("b_head", C.c_void_p),
                ("attention", C.c_int)]


def lib():
    """Load the built library (build it first if it was never built); fail loudly otherwise -- also when
    the binary on disk was compiled from other sources than the ones beside it (no silent rebuild)."""
    global _lib
    if _lib is None:
        from .build import build_library, source_id
        if not os.path.exists(LIB_PATH):
            build_library()
        loaded = C.CDLL(LIB_PATH)
        try:
            loaded.moe_build_id.restype = C.c_char_p
            built_from = loaded.moe_build_id().decode()
        except AttributeError:
            built_from = "none"
        if built_from != source_id():
            raise RuntimeError(
                f"{LIB_PATH} was built from sources {built_from}, the sources here are {source_id()}: rebuild it "
                "(python -m paper_2605_11537_amd.build)")
        _lib = loaded
        _lib.moe_last_error.restype = C.c_char_p
        for n in EXPORTS:
            f = getattr(_lib, n)
            if n.endswith("_bytes") or n.endswith("_flops"):
                f.restype = C.c_size_t
            elif n not in ("moe_last_error", "moe_build_id"):
                f.restype = C.c_int
        I, S, P = C.c_int, C.c_size_t, C.c_void_p
        _lib.moe_route_workspace_bytes.argtypes = [I, I, I, I]
        _lib.moe_route.argtypes = [P, P, I, P, I, I, I, I, P, P, P, P, S, P]
        _lib.sru_predict_workspace_bytes.argtypes = [C.POINTER(SruWeightsC), I, I, I]
        _lib.sru_predict.argtypes = [P, C.POINTER(SruWeightsC), I, I, I, P, P, P, S, P]
        _lib.replica_plan_workspace_bytes.argtypes = [I, I]
        _lib.replica_plan.argtypes = [P, I, I, I, I, I, P, P, P, P, P, P, S, P]
        _lib.moe_dispatch_workspace_bytes.argtypes = [I, I]
        _lib.moe_dispatch.argtypes = [P, P, P, I, I, I, I, I, I, P, P, P, P, P, P, P, P, S, P]
        _lib.moe_dispatch_static.argtypes = [P, P, P, I, I, I, I, I, I, P, P, P, P, P, P, P, P]
        _lib.moe_packed_weights_bytes.argtypes = [I, I, I, I]
        _lib.moe_pack_weights.argtypes = [P, I, I, I, I, P, P]
        _lib.moe_expert_ffn_workspace_bytes.argtypes = [I, I, I, I, I]
        _lib.moe_expert_ffn.argtypes = [P, P, P, P, I, P, P, P, I, I, I, I, I, I, I, P, P, S, P]
        _lib.moe_expert_ffn_timed.argtypes = [P, I, P, P, P, I, P, P, P, I, I, I, I, I, I, I, P, P, S, P, P, P, P]
        _lib.moe_combine.argtypes = [P, P, P, P, I, I, I, I, P, P]
        _lib.moe_route_topk.argtypes = [P, P, I, P, I, I, I, I, I, I, P, P, P, P, S, P]
        _lib.moe_dispatch_topk.argtypes = [P, P, P, I, I, I, I, I, I, I, P, P, P, P, P, P, P, P, P, S, P]
        _lib.moe_expert_ffn_rows.argtypes = [P, I, P, P, P, I, P, P, P, I, I, I, I, I, I, I, P, P, S, P]
        _lib.moe_combine_topk.argtypes = [P, P, P, P, I, I, I, I, I, P, P]
        _lib.moe_measure_sink_bytes.argtypes = []
        _lib.moe_measure_stream_read.argtypes = [P, S, I, I, P, P]
        _lib.moe_measure_mfma_bf16_flops.argtypes = [I]
        _lib.moe_measure_mfma_bf16.argtypes = [I, I, P, P]
        _lib.moe_plan_dispatch_workspace_bytes.argtypes = [I, I, I, I]
        _lib.moe_plan_dispatch.argtypes = [P, I, P, I, I, I, I, I, I] + [P] * 12 + [P, S, P]
    return _lib


def _check(rc: int):
    if rc != 0:
        raise MoeError(rc, lib().moe_last_error().decode())


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MOE_F32
    if t.dtype == torch.bfloat16:
        return MOE_BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _ptr(t):
    if t is None:
        return None
    if not (t.is_cuda and t.is_contiguous()):
        raise ValueError("device-resident contiguous tensors only")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _i32(n, dev):
    return torch.empty(n, dtype=torch.int32, device=dev)


def _ws(nbytes, dev):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=dev)


# --------------------------------------------------------------------------- the calls
def moe_route(x, w_router, b_router=None, want_logits=False, out=None, ws=None, w_layout=LAYOUT_PLAIN):
    """-> (expert_idx int32[T], expert_prob f32[T], logits f32[T,E] or None).  w_router is [d,E];
    with w_layout=LAYOUT_PACKED it is the image ``moe_pack_weights(w_router[None])[0]``."""
    T, d = x.shape
    E = w_router.shape[1]
    dev = x.device
    dt = _dt(x)
    if _dt(w_router) != dt or w_router.shape[0] != d:
        raise ValueError("w_router must be [d, E] (or its packed image) in the dtype of x")
    idx, prob = out if out is not None else (_i32(T, dev), torch.empty(T, dtype=torch.float32, device=dev))
    logits = torch.empty(T, E, dtype=torch.float32, device=dev) if want_logits else None
    need = lib().moe_route_workspace_bytes(T, d, E, dt)
    ws = ws if ws is not None else _ws(need, dev)
    _check(lib().moe_route(_ptr(x), _ptr(w_router), w_layout, _ptr(b_router), T, d, E, dt, _ptr(idx), _ptr(prob),
                           _ptr(logits), _ptr(ws), ws.numel(), _stream()))
    return idx, prob, logits


class SruWeights:
    """Holds the device tensors of an SRU predictor and the host-side C struct naming them."""

    def __init__(self, w_cat, b_f, b_r, w_head, b_head=None, pack=False, attention=False):
        """pack=True re-lays the (static) weights once with moe_pack_weights, so that sru_predict
        does not have to do it on every call (needs n_out = 128 or 256).  attention=True puts the
        sparsemax self-attention over the last layer's states in front of the head."""
        if pack:
            w_cat = [moe_pack_weights(w[None].contiguous())[0] for w in w_cat]
            w_head = moe_pack_weights(w_head[None].contiguous())[0]
        self.tensors = (list(w_cat), list(b_f) if b_f else None, list(b_r) if b_r else None, w_head, b_head)
        n = len(w_cat)
        self.n_layers = n
        self.n_in = w_cat[0].shape[0]
        self.n_hidden, self.n_out = w_head.shape
        PT = C.c_void_p * n
        self._wc = PT(*[w.data_ptr() for w in w_cat])
        self._bf = PT(*[(b.data_ptr() if b is not None else None) for b in b_f]) if b_f else None
        self._br = PT(*[(b.data_ptr() if b is not None else None) for b in b_r]) if b_r else None
        self.c = SruWeightsC(n, self.n_in, self.n_hidden, self.n_out, LAYOUT_PACKED if pack else LAYOUT_PLAIN,
                             C.cast(self._wc, C.POINTER(C.c_void_p)),
                             C.cast(self._bf, C.POINTER(C.c_void_p)) if self._bf else None,
                             C.cast(self._br, C.POINTER(C.c_void_p)) if self._br else None,
                             w_head.data_ptr(), b_head.data_ptr() if b_head is not None else None,
                             1 if attention else 0)


def sru_predict(emb, weights: SruWeights, want_logits=False, out=None, ws=None):
    """emb [B,L,n_in] -> (pred_idx int32[B*L], logits f32[B*L,n_out] or None)."""
    B, L, _ = emb.shape
    dev = emb.device
    dt = _dt(emb)
    pred = out if out is not None else _i32(B * L, dev)
    logits = torch.empty(B * L, weights.n_out, dtype=torch.float32, device=dev) if want_logits else None
    if ws is None:
        need = lib().sru_predict_workspace_bytes(C.byref(weights.c), B, L, dt)
        if need == 0:
            # the size query answers 0 for arguments the library rejects: make the call itself, with no
            # tensors, so that its validation names what is wrong
            _check(lib().sru_predict(None, C.byref(weights.c), B, L, dt, None, None, None, 0, None) or -2)
        ws = _ws(need, dev)
    _check(lib().sru_predict(_ptr(emb), C.byref(weights.c), B, L, dt, _ptr(pred), _ptr(logits), _ptr(ws),
                             ws.numel(), _stream()))
    return pred, logits


def replica_plan(idx, E, budget, slot_capacity, policy=0, out=None, ws=None):
    """-> dict(plan_counts[E], replicas[E], slot_base[E+1], slot_expert[E+budget], n_slots[1])."""
    dev = idx.device
    if ws is None:
        need = lib().replica_plan_workspace_bytes(idx.shape[0], E)
        ws = _ws(need, dev) if need else None
    o = out if out is not None else dict(plan_counts=_i32(E, dev), replicas=_i32(E, dev),
                                         slot_base=_i32(E + 1, dev), slot_expert=_i32(E + budget, dev),
                                         n_slots=_i32(1, dev))
    _check(lib().replica_plan(_ptr(idx), idx.shape[0], E, budget, slot_capacity, policy, _ptr(o["plan_counts"]),
                              _ptr(o["replicas"]), _ptr(o["slot_base"]), _ptr(o["slot_expert"]),
                              _ptr(o["n_slots"]), _ptr(ws), ws.numel() if ws is not None else 0, _stream()))
    return o


def moe_dispatch(x, expert_idx, replicas, E, slot_capacity, max_slots, out=None, ws=None, shape=None,
                 dtype=None):
    """-> dict(counts, kept, expert_offset, slot_offset, perm, inv, x_perm).  With x=None (give
    ``shape=(T, d)`` and ``dtype``) only the index tables are built and no rows are copied."""
    T, d = x.shape if x is not None else shape
    dev = expert_idx.device
    dt = _dt(x) if x is not None else (MOE_BF16 if dtype == torch.bfloat16 else MOE_F32)
    o = out if out is not None else dict(counts=_i32(E, dev), kept=_i32(E, dev), expert_offset=_i32(E + 1, dev),
                                         slot_offset=_i32(max_slots + 1, dev), perm=_i32(T, dev),
                                         inv=_i32(T, dev), x_perm=torch.empty_like(x) if x is not None else None)
    ws = ws if ws is not None else _ws(lib().moe_dispatch_workspace_bytes(T, E), dev)
    xp = o["x_perm"] if x is not None else None
    _check(lib().moe_dispatch(_ptr(x), _ptr(expert_idx), _ptr(replicas), T, d, E, slot_capacity, max_slots, dt,
                              _ptr(o["counts"]), _ptr(o["kept"]), _ptr(o["expert_offset"]), _ptr(o["slot_offset"]),
                              _ptr(o["perm"]), _ptr(o["inv"]), _ptr(xp), _ptr(ws), ws.numel(), _stream()))
    return o


def moe_dispatch_static(x, expert_idx, replicas, E, slot_capacity, max_slots, out, shape=None, dtype=None):
    """moe_dispatch without a workspace (the library's static scratch array): ``out`` must hold every
    output tensor (the dict of ``moe_dispatch``), so that nothing is allocated here either."""
    T, d = x.shape if x is not None else shape
    dt = _dt(x) if x is not None else (MOE_BF16 if dtype == torch.bfloat16 else MOE_F32)
    xp = out["x_perm"] if x is not None else None
    _check(lib().moe_dispatch_static(_ptr(x), _ptr(expert_idx), _ptr(replicas), T, d, E, slot_capacity, max_slots,
                                     dt, _ptr(out["counts"]), _ptr(out["kept"]), _ptr(out["expert_offset"]),
                                     _ptr(out["slot_offset"]), _ptr(out["perm"]), _ptr(out["inv"]), _ptr(xp),
                                     _stream()))
    return out


def moe_pack_weights(w, out=None):
    """[E,K,N] bf16 row-major -> packed image for the matrix-core kernels (same byte size)."""
    E, K, N = w.shape
    out = out if out is not None else torch.empty_like(w)
    _check(lib().moe_pack_weights(_ptr(w), E, K, N, _dt(w), _ptr(out), _stream()))
    return out


def moe_expert_ffn(x_perm, w1, w2, slot_offset, slot_expert, n_slots, E, F, max_slots=None,
                   schedule=SCHEDULE_SLOTS, weight_layout=None, out=None, ws=None, row_index=None, events=None):
    """-> y_perm [max_rows, d].  bf16 weights must already be packed (``moe_pack_weights``).
    With row_index (moe_dispatch's perm), x_perm is the unpermuted token matrix (fused gather).
    events (measurement only): three torch.cuda.Event objects (enable_timing=True, already created by a
    first record()) recorded before, between and after the two products (moe_expert_ffn_timed)."""
    max_rows, d = x_perm.shape
    dev = x_perm.device
    dt = _dt(x_perm)
    if weight_layout is None:
        weight_layout = LAYOUT_PACKED if dt == MOE_BF16 else LAYOUT_PLAIN
    if max_slots is None:
        max_slots = slot_expert.shape[0]
    y = out if out is not None else torch.empty_like(x_perm)
    ws = ws if ws is not None else _ws(lib().moe_expert_ffn_workspace_bytes(max_rows, max_slots, d, F, dt), dev)
    if events is not None:
        _check(lib().moe_expert_ffn_timed(_ptr(x_perm), max_rows, _ptr(row_index), _ptr(w1), _ptr(w2), weight_layout,
                                          _ptr(slot_offset), _ptr(slot_expert), _ptr(n_slots), max_rows, max_slots, E,
                                          d, F, dt, schedule, _ptr(y), _ptr(ws), ws.numel(), _stream(),
                                          *[C.c_void_p(e.cuda_event) for e in events]))
        return y
    _check(lib().moe_expert_ffn(_ptr(x_perm), _ptr(row_index), _ptr(w1), _ptr(w2), weight_layout, _ptr(slot_offset),
                                _ptr(slot_expert), _ptr(n_slots), max_rows, max_slots, E, d, F, dt, schedule,
                                _ptr(y), _ptr(ws), ws.numel(), _stream()))
    return y


def moe_combine(y_perm, x, inv, expert_prob, residual=0, out=None):
    T, d = x.shape
    o = out if out is not None else torch.empty_like(x)
    _check(lib().moe_combine(_ptr(y_perm), _ptr(x), _ptr(inv), _ptr(expert_prob), T, d, _dt(x), int(residual),
                             _ptr(o), _stream()))
    return o


def moe_plan_dispatch(plan_idx, expert_idx, E, budget, slot_capacity, policy=0, plan_out=None, disp_out=None,
                      ws=None):
    """replica_plan on plan_idx, then moe_dispatch's index tables for expert_idx ([T] or [k,T]) under
    that plan, in one call.  -> (plan dict, dispatch dict) with the keys of the separate calls
    (dispatch: no x_perm; row_token when expert_idx is [k,T])."""
    dev = expert_idx.device
    k = expert_idx.shape[0] if expert_idx.dim() == 2 else 1
    T = expert_idx.shape[-1]
    A = k * T
    max_slots = E + budget
    po = plan_out if plan_out is not None else dict(plan_counts=_i32(E, dev), replicas=_i32(E, dev),
                                                    slot_base=_i32(E + 1, dev), slot_expert=_i32(E + budget, dev),
                                                    n_slots=_i32(1, dev))
    do = disp_out if disp_out is not None else dict(
        counts=_i32(E, dev), kept=_i32(E, dev), expert_offset=_i32(E + 1, dev), slot_offset=_i32(max_slots + 1, dev),
        perm=_i32(A, dev), inv=_i32(A, dev).view(expert_idx.shape),
        row_token=_i32(A, dev) if expert_idx.dim() == 2 else None, x_perm=None)
    n_plan = plan_idx.numel()
    if ws is None:
        need = lib().moe_plan_dispatch_workspace_bytes(n_plan, T, k, E)
        ws = _ws(need, dev) if need else None
    _check(lib().moe_plan_dispatch(_ptr(plan_idx), n_plan, _ptr(expert_idx), T, k, E, budget, slot_capacity, policy,
                                   _ptr(po["plan_counts"]), _ptr(po["replicas"]), _ptr(po["slot_base"]),
                                   _ptr(po["slot_expert"]), _ptr(po["n_slots"]), _ptr(do["counts"]), _ptr(do["kept"]),
                                   _ptr(do["expert_offset"]), _ptr(do["slot_offset"]), _ptr(do["perm"]),
                                   _ptr(do["inv"]), _ptr(do.get("row_token")), _ptr(ws),
                                   ws.numel() if ws is not None else 0, _stream()))
    return po, do


# --------------------------------------------------------------------------- measurement
def measure_ceilings(read_bytes=1 << 30, mfma_iters=4000, repeats=5):
    """Event-timed ceilings of this machine for kernels shaped like the library's (see the header's
    measurement section): best of ``repeats`` launches each.  -> dict of GB/s and TFLOP/s."""
    dev = torch.device("cuda")
    L = lib()
    sink = torch.zeros(L.moe_measure_sink_bytes(), dtype=torch.uint8, device=dev)
    buf = torch.empty(read_bytes, dtype=torch.uint8, device=dev)
    buf.random_(0, 255)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]

    def best(launch):
        t = []
        for _ in range(repeats + 1):
            ev[0].record()
            _check(launch())
            ev[1].record()
            torch.cuda.synchronize()
            t.append(ev[0].elapsed_time(ev[1]))
        return min(t[1:]) * 1e-3

    st = _stream()
    out = {}
    for nt, name in ((0, "hbm_read_GBs"), (1, "hbm_read_nontemporal_GBs")):
        out[name] = round(read_bytes / best(lambda: L.moe_measure_stream_read(_ptr(buf), read_bytes, nt, 0, _ptr(sink), st)) / 1e9, 1)
    # one workgroup per compute unit on 1, 2, 144 units (128 KB in flight each): the per-CU stream rate, and
    # what a kernel with one workgroup per expert slot of the 144-slot workload could pull
    for wgs, name, nbytes in ((1, "one_workgroup_read_GBs", 1 << 26), (2, "two_workgroups_read_GBs", 1 << 26),
                              (144, "workgroups_144_read_GBs", read_bytes)):
        out[name] = round(nbytes / best(lambda: L.moe_measure_stream_read(_ptr(buf), nbytes, 1, wgs, _ptr(sink), st)) / 1e9, 1)
    flops = L.moe_measure_mfma_bf16_flops(mfma_iters)
    for fl, name in ((0, "mfma_bf16_registers_TFLOPs"), (1, "mfma_bf16_operands_from_lds_TFLOPs")):
        out[name] = round(flops / best(lambda: L.moe_measure_mfma_bf16(mfma_iters, fl, _ptr(sink), st)) / 1e12, 1)
    return out


# --------------------------------------------------------------------------- top-k routing
def moe_route_topk(x, w_router, b_router, k, renormalize=False, want_logits=False, out=None, ws=None,
                   w_layout=LAYOUT_PLAIN):
    """-> (expert_idx int32[k,T], expert_weight f32[k,T], logits f32[T,E] or None); choice-major."""
    T, d = x.shape
    E = w_router.shape[1]
    dev = x.device
    dt = _dt(x)
    if _dt(w_router) != dt or w_router.shape[0] != d:
        raise ValueError("w_router must be [d, E] (or its packed image) in the dtype of x")
    idx, wgt = out if out is not None else (_i32(k * T, dev).view(k, T),
                                            torch.empty(k, T, dtype=torch.float32, device=dev))
    logits = torch.empty(T, E, dtype=torch.float32, device=dev) if want_logits else None
    ws = ws if ws is not None else _ws(lib().moe_route_workspace_bytes(T, d, E, dt), dev)
    _check(lib().moe_route_topk(_ptr(x), _ptr(w_router), w_layout, _ptr(b_router), T, d, E, dt, int(k),
                                int(bool(renormalize)), _ptr(idx), _ptr(wgt), _ptr(logits), _ptr(ws), ws.numel(),
                                _stream()))
    return idx, wgt, logits


def moe_dispatch_topk(x, expert_idx, replicas, E, slot_capacity, max_slots, out=None, ws=None, shape=None,
                      dtype=None):
    """expert_idx int32[k,T] -> dict(counts, kept, expert_offset, slot_offset, perm[k*T], inv[k,T],
    row_token[k*T], x_perm [k*T,d] or None).  With x=None (give ``shape=(T, d)`` and ``dtype``) only
    the index tables are built."""
    k = expert_idx.shape[0]
    T, d = x.shape if x is not None else shape
    A = k * T
    dev = expert_idx.device
    dt = _dt(x) if x is not None else (MOE_BF16 if dtype == torch.bfloat16 else MOE_F32)
    o = out if out is not None else dict(
        counts=_i32(E, dev), kept=_i32(E, dev), expert_offset=_i32(E + 1, dev), slot_offset=_i32(max_slots + 1, dev),
        perm=_i32(A, dev), inv=_i32(A, dev).view(k, T), row_token=_i32(A, dev),
        x_perm=torch.empty(A, d, dtype=x.dtype, device=dev) if x is not None else None)
    ws = ws if ws is not None else _ws(lib().moe_dispatch_workspace_bytes(A, E), dev)
    xp = o["x_perm"] if x is not None else None
    _check(lib().moe_dispatch_topk(_ptr(x), _ptr(expert_idx), _ptr(replicas), T, k, d, E, slot_capacity, max_slots,
                                   dt, _ptr(o["counts"]), _ptr(o["kept"]), _ptr(o["expert_offset"]),
                                   _ptr(o["slot_offset"]), _ptr(o["perm"]), _ptr(o["inv"]), _ptr(o["row_token"]),
                                   _ptr(xp), _ptr(ws), ws.numel(), _stream()))
    return o


def moe_expert_ffn_rows(x, row_index, max_rows, w1, w2, slot_offset, slot_expert, n_slots, E, F, max_slots=None,
                        schedule=SCHEDULE_SLOTS, weight_layout=None, out=None, ws=None, events=None):
    """moe_expert_ffn gathering its rows from x [n_x_rows, d] through row_index [max_rows]
    (moe_dispatch_topk's row_token).  -> y_perm [max_rows, d]."""
    n_x_rows, d = x.shape
    dev = x.device
    dt = _dt(x)
    if weight_layout is None:
        weight_layout = LAYOUT_PACKED if dt == MOE_BF16 else LAYOUT_PLAIN
    if max_slots is None:
        max_slots = slot_expert.shape[0]
    y = out if out is not None else torch.empty(max_rows, d, dtype=x.dtype, device=dev)
    ws = ws if ws is not None else _ws(lib().moe_expert_ffn_workspace_bytes(max_rows, max_slots, d, F, dt), dev)
    args = (_ptr(x), n_x_rows, _ptr(row_index), _ptr(w1), _ptr(w2), weight_layout, _ptr(slot_offset),
            _ptr(slot_expert), _ptr(n_slots), max_rows, max_slots, E, d, F, dt, schedule, _ptr(y), _ptr(ws),
            ws.numel(), _stream())
    if events is not None:
        _check(lib().moe_expert_ffn_timed(*args, *[C.c_void_p(e.cuda_event) for e in events]))
    else:
        _check(lib().moe_expert_ffn_rows(*args))
    return y


def moe_combine_topk(y_perm, x, inv, expert_weight, residual=0, out=None):
    """inv int32[k,T], expert_weight f32[k,T] -> out [T,d]."""
    T, d = x.shape
    k = inv.shape[0]
    o = out if out is not None else torch.empty_like(x)
    _check(lib().moe_combine_topk(_ptr(y_perm), _ptr(x), _ptr(inv), _ptr(expert_weight), T, k, d, _dt(x),
                                  int(residual), _ptr(o), _stream()))
    return o


class MoeLayerTopK:
    """The top-k layer: route_topk -> plan over the k*T ids -> dispatch_topk -> expert FFN (rows
    gathered through row_token) -> combine_topk.  Preallocated buffers, pure sequencing."""

    def __init__(self, T, d, F, E, k, budget, slot_capacity, dtype, device="cuda", policy=0, renormalize=False):
        self.T, self.d, self.F, self.E, self.k, self.R, self.C = T, d, F, E, k, budget, slot_capacity
        self.policy, self.renormalize = policy, renormalize
        self.max_slots = E + budget
        A = k * T
        dev = torch.device(device)
        dt = MOE_BF16 if dtype == torch.bfloat16 else MOE_F32
        L = lib()
        self.route_out = (_i32(A, dev).view(k, T), torch.empty(k, T, dtype=torch.float32, device=dev))
        self.route_ws = _ws(L.moe_route_workspace_bytes(T, d, E, dt), dev)
        self.plan_out = dict(plan_counts=_i32(E, dev), replicas=_i32(E, dev), slot_base=_i32(E + 1, dev),
                             slot_expert=_i32(E + budget, dev), n_slots=_i32(1, dev))
        self.disp_out = dict(counts=_i32(E, dev), kept=_i32(E, dev), expert_offset=_i32(E + 1, dev),
                             slot_offset=_i32(self.max_slots + 1, dev), perm=_i32(A, dev),
                             inv=_i32(A, dev).view(k, T), row_token=_i32(A, dev), x_perm=None)
        self.front_ws = _ws(L.moe_plan_dispatch_workspace_bytes(A, T, k, E), dev)
        self.y_perm = torch.zeros(A, d, dtype=dtype, device=dev)
        self.ffn_ws = _ws(L.moe_expert_ffn_workspace_bytes(A, self.max_slots, d, F, dt), dev)
        self.out = torch.empty(T, d, dtype=dtype, device=dev)

    def forward(self, x, w_router, b_router, w1, w2, plan_ids=None, schedule=SCHEDULE_SLOTS, residual=0,
                out=None, router_layout=LAYOUT_PLAIN, marks=None, ffn_events=None):
        """marks, ffn_events: as in MoeLayer.forward."""
        if marks is not None:
            marks[0].record()
        idx, wgt, _ = moe_route_topk(x, w_router, b_router, self.k, self.renormalize, out=self.route_out,
                                     ws=self.route_ws, w_layout=router_layout)
        if marks is not None:
            marks[1].record()
        pl, dp = moe_plan_dispatch(idx.view(-1) if plan_ids is None else plan_ids, idx, self.E, self.R, self.C,
                                   self.policy, plan_out=self.plan_out, disp_out=self.disp_out, ws=self.front_ws)
        if marks is not None:
            marks[2].record()
        y = moe_expert_ffn_rows(x, dp["row_token"], self.k * self.T, w1, w2, dp["slot_offset"], pl["slot_expert"],
                                pl["n_slots"], self.E, self.F, max_slots=self.max_slots, schedule=schedule,
                                out=self.y_perm, ws=self.ffn_ws, events=ffn_events)
        if marks is not None:
            marks[3].record()
        o = moe_combine_topk(y, x, dp["inv"], wgt, residual, out=self.out if out is None else out)
        if marks is not None:
            marks[4].record()
        return o


# --------------------------------------------------------------------------- whole layer
class MoeLayer:
    """Preallocated buffers + the chain route -> plan -> dispatch -> expert FFN -> combine for
    one layer shape.  Pure sequencing of the calls above on the current stream."""

    def __init__(self, T, d, F, E, budget, slot_capacity, dtype, device="cuda", policy=0):
        self.T, self.d, self.F, self.E, self.R, self.C = T, d, F, E, budget, slot_capacity
        self.policy = policy
        self.max_slots = E + budget
        dev = torch.device(device)
        dt = MOE_BF16 if dtype == torch.bfloat16 else MOE_F32
        L = lib()
        self.route_out = (_i32(T, dev), torch.empty(T, dtype=torch.float32, device=dev))
        self.route_ws = _ws(L.moe_route_workspace_bytes(T, d, E, dt), dev)
        self.plan_out = dict(plan_counts=_i32(E, dev), replicas=_i32(E, dev), slot_base=_i32(E + 1, dev),
                             slot_expert=_i32(E + budget, dev), n_slots=_i32(1, dev))
        self.plan_ws = _ws(L.replica_plan_workspace_bytes(T, E), dev)
        self.disp_out = dict(counts=_i32(E, dev), kept=_i32(E, dev), expert_offset=_i32(E + 1, dev),
                             slot_offset=_i32(self.max_slots + 1, dev), perm=_i32(T, dev), inv=_i32(T, dev),
                             x_perm=torch.zeros(T, d, dtype=dtype, device=dev))
        self.disp_ws = _ws(L.moe_dispatch_workspace_bytes(T, E), dev)
        self.front_ws = _ws(L.moe_plan_dispatch_workspace_bytes(T, T, 1, E), dev)
        self.y_perm = torch.zeros(T, d, dtype=dtype, device=dev)
        self.ffn_ws = _ws(L.moe_expert_ffn_workspace_bytes(T, self.max_slots, d, F, dt), dev)
        self.out = torch.empty(T, d, dtype=dtype, device=dev)

    def forward(self, x, w_router, b_router, w1, w2, plan_ids=None, schedule=SCHEDULE_SLOTS, residual=0,
                out=None, router_layout=LAYOUT_PLAIN, fuse_gather=True, plan=None, marks=None, ffn_events=None):
        """plan: tables of a replica_plan call made earlier (e.g. by MoePipeline on another stream);
        otherwise the plan is computed here from plan_ids, or from the router's own ids.
        marks: five torch.cuda.Event objects recorded before the router and after each of the four
        calls (router, plan + dispatch, expert FFN, combine), for per-call timing.
        ffn_events: three events recorded around the two products of the expert FFN (measurement only)."""
        if marks is not None:
            marks[0].record()
        idx, prob, _ = moe_route(x, w_router, b_router, out=self.route_out, ws=self.route_ws,
                                 w_layout=router_layout)
        if marks is not None:
            marks[1].record()
        R = self.R
        if plan is None and fuse_gather:
            pl, dp = moe_plan_dispatch(idx if plan_ids is None else plan_ids, idx, self.E, R, self.C, self.policy,
                                       plan_out=self.plan_out, disp_out=self.disp_out, ws=self.front_ws)
        else:
            pl = plan if plan is not None else replica_plan(idx if plan_ids is None else plan_ids, self.E, R,
                                                            self.C, self.policy, out=self.plan_out, ws=self.plan_ws)
            dp = moe_dispatch(None if fuse_gather else x, idx, pl["replicas"], self.E, self.C, self.max_slots,
                              out=self.disp_out, ws=self.disp_ws, shape=(self.T, self.d), dtype=x.dtype)
        if marks is not None:
            marks[2].record()
        y = moe_expert_ffn(x if fuse_gather else dp["x_perm"], w1, w2, dp["slot_offset"], pl["slot_expert"],
                           pl["n_slots"], self.E, self.F, max_slots=self.max_slots, schedule=schedule,
                           out=self.y_perm, ws=self.ffn_ws, row_index=dp["perm"] if fuse_gather else None,
                           events=ffn_events)
        if marks is not None:
            marks[3].record()
        o = moe_combine(y, x, dp["inv"], prob, residual, out=self.out if out is None else out)
        if marks is not None:
            marks[4].record()
        return o


class MoePipeline:
    """Predictor and replica plan of batch i+1 on a second stream while the layer of batch i runs
    (the paper's two threads and their queue of per-batch tables, as two HIP streams and two sets of
    plan tables).  ``predict(emb)`` enqueues sru_predict + replica_plan for the next batch;
    ``forward(x, ...)`` runs the layer of the oldest batch predicted and not yet run.  The embeddings
    must be ready when predict is called (they are not ordered after work on the layer's stream).
    Both streams have the default priority."""

    def __init__(self, layer: "MoeLayer", sru_weights, B, L):
        self.layer, self.w, self.B, self.L = layer, sru_weights, B, L
        dev = layer.out.device
        E, R, T = layer.E, layer.R, layer.T
        self.stream = torch.cuda.Stream(device=dev)
        self.sets = []
        for _ in range(2):
            plan = dict(plan_counts=_i32(E, dev), replicas=_i32(E, dev), slot_base=_i32(E + 1, dev),
                        slot_expert=_i32(E + R, dev), n_slots=_i32(1, dev))
            self.sets.append(dict(plan=plan, ids=_i32(T, dev), ready=torch.cuda.Event(), free=torch.cuda.Event()))
        self.sru_ws = _ws(lib().sru_predict_workspace_bytes(C.byref(sru_weights.c), B, L, MOE_BF16), dev)
        self.plan_ws = _ws(lib().replica_plan_workspace_bytes(T, E), dev)
        self.n_pred = self.n_run = 0

    def predict(self, emb):
        if self.n_pred - self.n_run >= 2:
            raise RuntimeError("two batches are already predicted and waiting for their layer")
        s = self.sets[self.n_pred % 2]
        with torch.cuda.stream(self.stream):
            self.stream.wait_event(s["free"])      # the layer that last read these tables has finished
            ids, _ = sru_predict(emb, self.w, out=s["ids"], ws=self.sru_ws)
            replica_plan(ids, self.layer.E, self.layer.R, self.layer.C, self.layer.policy, out=s["plan"],
                         ws=self.plan_ws)
            s["ready"].record(self.stream)
        self.n_pred += 1

    def forward(self, x, w_router, b_router, w1, w2, **kw):
        if self.n_run >= self.n_pred:
            raise RuntimeError("no predicted batch is waiting")
        s = self.sets[self.n_run % 2]
        main = torch.cuda.current_stream()
        main.wait_event(s["ready"])
        out = self.layer.forward(x, w_router, b_router, w1, w2, plan=s["plan"], **kw)
        s["free"].record(main)
        self.n_run += 1
        return out
