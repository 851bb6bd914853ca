"""GPU parity of the top-k routing path against the oracle (``oracle/topk.py`` states the reading):
moe_route_topk, moe_dispatch_topk, moe_expert_ffn_rows, moe_combine_topk and the whole layer,
through the C ABI.  Integer tables bit for bit; floats within the tolerances of gpu_util."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import assert_close, f64, to_dev, to_host
from oracle import topk as otopk

pytestmark = pytest.mark.gpu


def _check_choices(g_idx, g_w, ref, tau, renormalize, what, wtol=1e-4):
    """Ids and their order equal the oracle's wherever every gap among the k+1 largest logits
    exceeds tau; elsewhere every choice must be a near-tie of the oracle's choice at its place.
    Weights are held against the softmax of the oracle's logits at the ids the GPU chose."""
    k, T = g_idx.shape
    clear = ref["gap"] > tau
    assert (g_idx[:, clear] == ref["idx"][:, clear]).all(), f"{what}: ids differ outside near-ties"
    l = ref["logits"]
    rows = np.arange(T)
    for j in range(k):
        assert np.abs(l[rows, g_idx[j]] - l[rows, ref["idx"][j]]).max() <= tau, f"{what}: choice {j}"
    srt = np.sort(g_idx, axis=0)
    assert (np.diff(srt, axis=0) > 0).all(), f"{what}: repeated expert in a token's choices"
    z = np.exp(l - l.max(axis=1, keepdims=True))
    p = z / z.sum(axis=1, keepdims=True)
    want = p[rows[None, :], g_idx]
    if renormalize:
        want = want / want.sum(axis=0, keepdims=True)
    assert np.abs(g_w - want).max() <= wtol, f"{what}: weights off by {np.abs(g_w - want).max():.2e}"
    return int((~clear).sum())


@pytest.mark.parametrize("T,d,E,dtype,k,renorm", [
    (1000, 128, 128, synth.BF16, 3, False),      # matrix-core router, ragged last tile
    (9000, 256, 256, synth.BF16, 2, True),       # its two-row-block build
    (16384 + 45, 256, 256, synth.BF16, 3, True),  # persistent router with the matrix in registers, ragged last tile
    (20000, 768, 256, synth.BF16, 2, False),     # the same at the benchmark's width
    (333, 128, 128, synth.BF16, 8, True),        # k at the limit
    (500, 64, 12, synth.F32, 3, False),          # generic router, fp32
    (257, 40, 70, synth.BF16, 5, True),          # generic router, E over one wavefront
    (64, 16, 3, synth.F32, 3, True),             # k = E
])
def test_route_topk(T, d, E, dtype, k, renorm):
    import paper_2605_11537_amd as moe
    x = synth.normal_tensor((T, d), 1.0, [71, T], dtype)
    wr = synth.normal_tensor((d, E), 0.3, [72, E], dtype)
    b = (np.random.default_rng(73).standard_normal(E) * 0.1).astype(np.float32)
    wr[:, 5 % E] = wr[:, 1 % E]                                  # two experts with equal logits
    b[5 % E] = b[1 % E]
    ref = oracle.route_topk(x, wr, b, k, renorm)
    idx, w, logits = moe.moe_route_topk(to_dev(x), to_dev(wr), to_dev(b), k, renorm, want_logits=True)
    tau = 1e-4 * max(1.0, np.abs(ref["logits"]).max())
    lerr = np.abs(to_host(logits) - ref["logits"]).max()
    assert lerr <= tau
    # a logit error e moves a softmax weight by at most 2e (relative), the renormalised one by 4e
    flips = _check_choices(to_host(idx), to_host(w), ref, tau, renorm, "route_topk", wtol=2e-6 + 4 * lerr)
    print(f"route_topk T={T} E={E} k={k}: {flips} tokens with a near-tie, logit error {lerr:.2e}", flush=True)
    # the equal pair: the lower id comes first whenever both are chosen
    gi = to_host(idx)
    if E > 5:
        both = (gi == 1).any(axis=0) & (gi == 5).any(axis=0)
        pos1 = np.argmax(gi == 1, axis=0)
        pos5 = np.argmax(gi == 5, axis=0)
        assert (pos1[both] + 1 == pos5[both]).all()
    # first choice = the top-1 router, bit for bit; packed router weights give the same results
    i1, p1, _ = moe.moe_route(to_dev(x), to_dev(wr), to_dev(b))
    ik, wk, _ = moe.moe_route_topk(to_dev(x), to_dev(wr), to_dev(b), 1)
    assert torch.equal(i1, ik[0]) and torch.equal(p1, wk[0])
    assert torch.equal(i1, idx[0])
    if dtype == synth.BF16 and E in (128, 256):
        wp = moe.moe_pack_weights(to_dev(wr)[None].contiguous())[0]
        i2, w2, _ = moe.moe_route_topk(to_dev(x), wp, to_dev(b), k, renorm, w_layout=moe.LAYOUT_PACKED)
        assert torch.equal(i2, idx) and torch.equal(w2, w)


def _topk_ids(T, E, k, seed, s=1.1):
    """Distinct ids per token, skewed: Zipf scores plus noise, k largest."""
    rng = np.random.default_rng(seed)
    score = np.log(synth.zipf_weights(E, s))[None, :] + rng.gumbel(size=(T, E))
    return np.ascontiguousarray(np.argsort(-score, axis=1)[:, :k].T.astype(np.int32))


@pytest.mark.parametrize("T,d,E,k,C,R,dtype", [
    (3000, 64, 16, 3, 400, 6, synth.BF16),       # several 1024-entry blocks, ragged, capacity binds
    (700, 32, 8, 2, 60, 0, synth.F32),           # no replicas
    (1, 16, 4, 3, 1, 2, synth.F32),              # one token
])
def test_dispatch_topk(T, d, E, k, C, R, dtype):
    import paper_2605_11537_amd as moe
    ids = _topk_ids(T, E, k, 81 + T)
    x = synth.normal_tensor((T, d), 1.0, [82, T], dtype)
    pl = oracle.plan(ids.reshape(-1), E, R, C)
    ref = oracle.dispatch(otopk.assignment_rows(x, k), ids.reshape(-1), pl["replicas"], E, C, E + R)
    got = moe.moe_dispatch_topk(to_dev(x), to_dev(ids), to_dev(pl["replicas"]), E, C, E + R)
    for name in ("counts", "kept", "expert_offset", "slot_offset", "perm"):
        assert (to_host(got[name]) == ref[name]).all(), name
    assert (to_host(got["inv"]).reshape(-1) == ref["inv"]).all()
    K = int(ref["expert_offset"][E])
    if T > 1:
        assert K < k * T                                         # something was dropped
    want_tok = np.where(ref["perm"] >= 0, ref["perm"] % T, -1)
    assert (to_host(got["row_token"]) == want_tok).all()
    assert (to_host(got["x_perm"])[:K] == ref["x_perm"][:K]).all()
    # tables only
    got2 = moe.moe_dispatch_topk(None, to_dev(ids), to_dev(pl["replicas"]), E, C, E + R, shape=(T, d),
                                 dtype=torch.bfloat16 if dtype == synth.BF16 else torch.float32)
    assert torch.equal(got2["row_token"], got["row_token"]) and torch.equal(got2["inv"], got["inv"])


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
@pytest.mark.parametrize("residual", [0, 1])
def test_combine_topk(dtype, residual):
    import paper_2605_11537_amd as moe
    k, T, d, rows = 3, 1500, 72 if dtype == synth.F32 else 136, 3100
    rng = np.random.default_rng(91)
    x = synth.normal_tensor((T, d), 1.0, [92], dtype)
    y = synth.normal_tensor((rows, d), 1.0, [93], dtype)
    inv = np.full(k * T, -1, np.int32)
    kept = rng.permutation(k * T)[:rows]
    inv[kept] = rng.permutation(rows).astype(np.int32)
    inv = inv.reshape(k, T)
    inv[:, ::50] = -1                                            # tokens with no kept choice
    w = rng.random((k, T)).astype(np.float32)
    ref = oracle.combine_topk(y, x, inv, w, residual)
    got = to_host(moe.moe_combine_topk(to_dev(y), to_dev(x), to_dev(inv), to_dev(w), residual))
    assert_close(got, ref, dtype, "combine_topk")
    none = (inv < 0).all(axis=0)
    assert none.sum() >= T // 50 and (got[none] == x[none]).all()
    # k = 1 is the top-1 combine
    a = moe.moe_combine_topk(to_dev(y), to_dev(x), to_dev(inv[:1].copy()), to_dev(w[:1].copy()), residual)
    b = moe.moe_combine(to_dev(y), to_dev(x), to_dev(inv[0].copy()), to_dev(w[0].copy()), residual)
    assert torch.equal(a, b)


@pytest.mark.parametrize("T,d,F,E,k,C,R,dtype,renorm,residual", [
    (1000, 128, 256, 8, 3, 300, 4, synth.BF16, False, 1),
    (777, 128, 256, 16, 2, 80, 5, synth.BF16, True, 0),
    (600, 64, 128, 8, 3, 200, 3, synth.F32, True, 1),
])
def test_layer_topk(T, d, F, E, k, C, R, dtype, renorm, residual):
    import paper_2605_11537_amd as moe
    c = synth.moe_layer_inputs(T, d, F, E, dtype, 1.2, 101 + T)
    tdt = torch.bfloat16 if dtype == synth.BF16 else torch.float32
    layer = moe.MoeLayerTopK(T, d, F, E, k, R, C, tdt, renormalize=renorm)
    w1, w2 = to_dev(c["w1"]), to_dev(c["w2"])
    if dtype == synth.BF16:
        w1, w2 = moe.moe_pack_weights(w1), moe.moe_pack_weights(w2)
    out = layer.forward(to_dev(c["x"]), to_dev(c["w_router"]), to_dev(c["b_router"]), w1, w2, residual=residual)
    torch.cuda.synchronize()
    g_idx, g_w = to_host(layer.route_out[0]), to_host(layer.route_out[1])
    rt = oracle.route_topk(c["x"], c["w_router"], c["b_router"], k, renorm)
    tau = 1e-4 * max(1.0, np.abs(rt["logits"]).max())
    _check_choices(g_idx, g_w, rt, tau, renorm, "layer route")
    # the oracle follows the GPU's routing decision from here on
    ref = oracle.layer_topk(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"], k, C, R, renormalize=renorm,
                            residual=residual, idx=g_idx, weight=g_w)
    for name, rk in (("plan_counts", "counts"), ("replicas", "replicas"), ("slot_expert", "slot_expert")):
        assert (to_host(layer.plan_out[name]) == ref["plan"][rk]).all(), name
    for name in ("kept", "expert_offset", "slot_offset", "perm"):
        assert (to_host(layer.disp_out[name]) == ref["dispatch"][name]).all(), name
    assert (to_host(layer.disp_out["inv"]).reshape(-1) == ref["dispatch"]["inv"]).all()
    K = int(ref["dispatch"]["expert_offset"][E])
    assert 0 < K < k * T and ref["plan"]["replicas"].max() > 1    # capacity binds, replicas granted
    assert_close(to_host(layer.y_perm)[:K], ref["y_perm"][:K], dtype, "y_perm")
    assert_close(to_host(out), ref["out"], dtype, "out")
    # the row gather equals the materialised rows
    dp = moe.moe_dispatch_topk(to_dev(c["x"]), layer.route_out[0], layer.plan_out["replicas"], E, C, E + R)
    y2 = moe.moe_expert_ffn(dp["x_perm"], w1, w2, dp["slot_offset"], layer.plan_out["slot_expert"],
                            layer.plan_out["n_slots"], E, F, max_slots=E + R)
    assert torch.equal(y2[:K], layer.y_perm[:K])


@pytest.mark.timeout(600)
def test_layer_top3_full_size():
    """The bench's top-3 workload (Switch-base-128 shapes, k = 3) in its launch configuration:
    integer tables at full size against the oracle fed the GPU's ids; sampled rows and tokens for
    the floats."""
    import paper_2605_11537_amd as moe
    c = synth.config_inputs(2)
    T, d, F, E, R, k = c["T"], c["d"], c["F"], c["E"], c["R"], 3
    C = k * c["C"]
    layer = moe.MoeLayerTopK(T, d, F, E, k, R, C, torch.bfloat16)
    x, b = to_dev(c["x"]), to_dev(c["b_router"])
    wr = moe.moe_pack_weights(to_dev(c["w_router"])[None].contiguous())[0]
    w1, w2 = moe.moe_pack_weights(to_dev(c["w1"])), moe.moe_pack_weights(to_dev(c["w2"]))
    out = to_host(layer.forward(x, wr, b, w1, w2, router_layout=moe.LAYOUT_PACKED))
    g_idx, g_w = to_host(layer.route_out[0]), to_host(layer.route_out[1])
    rt = oracle.route_topk(c["x"], c["w_router"], c["b_router"], k)
    tau = 1e-4 * max(1.0, np.abs(rt["logits"]).max())
    _check_choices(g_idx, g_w, rt, tau, False, "top-3 route")
    ids = g_idx.reshape(-1)
    pl = oracle.plan(ids, E, R, C)
    for name, rk in (("plan_counts", "counts"), ("replicas", "replicas"), ("slot_base", "slot_base"),
                     ("slot_expert", "slot_expert")):
        assert (to_host(layer.plan_out[name]) == pl[rk]).all(), name
    dp = oracle.dispatch(np.zeros((k * T, 4), np.float32), ids, pl["replicas"], E, C, E + R)
    for name in ("counts", "kept", "expert_offset", "slot_offset", "perm"):
        assert (to_host(layer.disp_out[name]) == dp[name]).all(), name
    inv = dp["inv"].reshape(k, T)
    assert (to_host(layer.disp_out["inv"]) == inv).all()
    K = int(dp["expert_offset"][E])
    # sampled tokens: all their kept rows are evaluated by the oracle
    rng = np.random.default_rng(12)
    dropped_any = np.where((inv < 0).any(axis=0))[0]
    toks = np.unique(np.concatenate([rng.choice(T, 40, replace=False), dropped_any[:8], [0, T - 1]]))
    rows = inv[:, toks].reshape(-1)
    rows = np.unique(rows[rows >= 0]).astype(np.int32)
    xp = np.zeros((k * T, d), np.uint16)
    xp[rows] = c["x"][dp["perm"][rows] % T]
    y = oracle.ffn(xp, c["w1"], c["w2"], dp["slot_offset"], pl["slot_expert"], pl["n_slots"], rows=rows)
    assert_close(to_host(layer.y_perm)[rows], y[rows], synth.BF16, "y_perm sample")
    ref_out = oracle.combine_topk(y, c["x"], inv, g_w, 0)
    assert_close(out[toks], ref_out[toks], synth.BF16, "out sample")
    none = (inv < 0).all(axis=0)
    assert (out[none] == c["x"][none]).all()
    print(f"top-3: kept {K}/{k * T}, slots {pl['n_slots']}, tokens with a dropped choice {dropped_any.size}",
          flush=True)
