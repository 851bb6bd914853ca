"""Full-size GPU parity on the large workloads, in the launch configuration bench.py times.

Integer stages (plan, dispatch) are compared bit for bit against the oracle fed the GPU's own router
ids; the float stages are compared on every kept row and every token (the oracle evaluates the whole
layer: a second or so at 16384 tokens, several seconds per layer at 65536); size-independent properties
(conservation, no drops, passthrough, slot schedule == expert schedule bit for bit) are checked as well.
"""
import time

import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import assert_close, check_ids_margin, f64, to_dev, to_host

pytestmark = pytest.mark.gpu


def _integer_parity(moe, layer, idx_host, E, C, R, T, plan_ids=None):
    pl = oracle.plan(idx_host if plan_ids is None else plan_ids, E, R, C)
    for k, rk in (("plan_counts", "counts"), ("replicas", "replicas"), ("slot_base", "slot_base"),
                  ("slot_expert", "slot_expert")):
        assert (to_host(layer.plan_out[k]) == pl[rk]).all(), k
    dp = oracle.dispatch(np.zeros((T, 4), np.float32), idx_host, pl["replicas"], E, C, E + R)
    for k in ("counts", "kept", "expert_offset", "slot_offset", "perm", "inv"):
        assert (to_host(layer.disp_out[k]) == dp[k]).all(), k
    return pl, dp


def _assert_rows_close(got, ref, what):
    """Element-wise bound, so that one bad row cannot hide behind the tensor's maximum: half a bf16 ulp
    of the value for its one rounding, plus accumulation-order noise relative to the tensor's scale."""
    g, r = f64(got), f64(ref)
    bad = np.abs(g - r) > 2.0 ** -7 * np.abs(r) + 1e-3 * np.abs(r).max()
    assert not bad.any(), f"{what}: {int(bad.sum())} elements off, first at row {int(np.argwhere(bad)[0][0])}"


@pytest.mark.timeout(600)
@pytest.mark.parametrize("cap_key", ["C", "C_alt"])
def test_workload4_full_size(cap_key):
    import paper_2605_11537_amd as moe
    t0 = time.time()
    c = synth.config_inputs(4)
    T, d, F, E, R, C = c["T"], c["d"], c["F"], c["E"], c["R"], c[cap_key]
    print(f"workload 4 C={C}: inputs in {time.time() - t0:.1f}s", flush=True)
    layer = moe.MoeLayer(T, d, F, E, R, C, torch.bfloat16)
    x, b = to_dev(c["x"]), to_dev(c["b_router"])
    wr = moe.moe_pack_weights(to_dev(c["w_router"])[None].contiguous())[0]
    w1, w2 = moe.moe_pack_weights(to_dev(c["w1"])), moe.moe_pack_weights(to_dev(c["w2"]))
    out = layer.forward(x, wr, b, w1, w2, router_layout=moe.LAYOUT_PACKED).clone()
    torch.cuda.synchronize()
    g_idx, g_prob = to_host(layer.route_out[0]), to_host(layer.route_out[1])
    rt = oracle.route(c["x"], c["w_router"], c["b_router"])
    tau = 1e-4 * max(1.0, np.abs(rt["logits"]).max())
    flips = check_ids_margin(g_idx, rt["idx"], rt["idx2"], rt["margin"], tau, "workload 4 route")
    same = g_idx == rt["idx"]
    assert np.abs(g_prob - rt["prob"])[same].max() <= 1e-4
    pl, dp = _integer_parity(moe, layer, g_idx, E, C, R, T)
    K = int(dp["expert_offset"][E])
    assert K + int((dp["inv"] < 0).sum()) == T
    got = to_host(out)
    dropped = dp["inv"] < 0
    assert (got[dropped] == c["x"][dropped]).all()
    # every kept row of the expert products and every token of the output
    xp = np.zeros_like(c["x"])
    xp[:K] = c["x"][dp["perm"][:K]]
    y = oracle.ffn(xp, c["w1"], c["w2"], dp["slot_offset"], pl["slot_expert"], pl["n_slots"])
    assert_close(to_host(layer.y_perm)[:K], y[:K], synth.BF16, "y_perm")
    _assert_rows_close(to_host(layer.y_perm)[:K], y[:K], "y_perm")
    ref_out = oracle.combine(y, c["x"], dp["inv"], g_prob, 0)
    assert_close(got, ref_out, synth.BF16, "out")
    # replication off (same plan): identical outputs
    out_off = layer.forward(x, wr, b, w1, w2, schedule=moe.SCHEDULE_EXPERTS, router_layout=moe.LAYOUT_PACKED)
    assert torch.equal(out, out_off)
    print(f"workload 4 C={C}: kept {K}/{T}, slots {pl['n_slots']}, {flips} near-tie flips, "
          f"total {time.time() - t0:.1f}s", flush=True)


@pytest.mark.timeout(900)
def test_workload5_stack_full_size():
    """6-layer stack, T=65536, E=256, one expert at 50% load, nothing may drop.  The oracle follows the
    whole batch through all six layers from its own state (the GPU contributes only the router's integer
    decision and probability of each layer, which are checked first); every token of every layer's
    output is compared, layer 0 also on every row of the second expert product.  Each layer is run a
    second time with the expert schedule (the 128-column kernel alone) and must agree bit for bit with the
    slot schedule (the persistent 256 x 256 tile kernel at this size) on all rows."""
    import paper_2605_11537_amd as moe
    t0 = time.time()
    c = synth.config_inputs(5, weights=False)
    T, d, F, E, R, C, NL = c["T"], c["d"], c["F"], c["E"], c["R"], c["C"], c["n_layers"]
    seed = synth.workloads.SEED0 + 5
    layer = moe.MoeLayer(T, d, F, E, R, C, torch.bfloat16)
    ref_x = c["x"].copy()                              # oracle-side state of the whole batch
    cur = to_dev(c["x"])
    nxt = torch.empty_like(cur)
    nxt_off = torch.empty_like(cur)
    most_slots = 0
    for l in range(NL):
        lay = c["layers"][l]
        w1h = synth.normal_tensor((E, d, F), 0.02, [seed, 50 + l], synth.BF16)
        w2h = synth.normal_tensor((E, F, d), 0.02, [seed, 60 + l], synth.BF16)
        w1, w2 = moe.moe_pack_weights(to_dev(w1h)), moe.moe_pack_weights(to_dev(w2h))
        wr = to_dev(lay["w_router"])
        layer.forward(cur, wr, None, w1, w2, residual=1, out=nxt)
        torch.cuda.synchronize()
        y_on = layer.y_perm.clone()
        g_idx, g_prob = to_host(layer.route_out[0]), to_host(layer.route_out[1])
        pl, dp = _integer_parity(moe, layer, g_idx, E, C, R, T)
        assert int(dp["expert_offset"][E]) == T and (dp["inv"] >= 0).all()      # nothing drops
        n = dp["counts"]
        assert n.max() >= 0.49 * T                                              # the hot expert
        most_slots = max(most_slots, int(pl["replicas"].max()))
        layer.forward(cur, wr, None, w1, w2, residual=1, out=nxt_off, schedule=moe.SCHEDULE_EXPERTS)
        torch.cuda.synchronize()
        assert torch.equal(y_on, layer.y_perm), f"layer {l}: tile kernel and 128-column kernel disagree"
        assert torch.equal(nxt, nxt_off)
        # the oracle on its own state: router decision first, then the layer under the GPU's ids
        rt = oracle.route(ref_x, lay["w_router"], None)
        tau = 1e-4 * max(1.0, np.abs(rt["logits"]).max())
        flips = check_ids_margin(g_idx, rt["idx"], rt["idx2"], rt["margin"], tau, f"layer {l} route")
        same = g_idx == rt["idx"]
        # layer 0 reads the same bits on both sides; later layers read states that differ by the bf16
        # roundings accumulated so far, so their gate probabilities agree less closely
        assert np.abs(g_prob - rt["prob"])[same].max() <= (1e-4 if l == 0 else 1e-2)
        xp = ref_x[dp["perm"]]
        y = oracle.ffn(xp, w1h, w2h, dp["slot_offset"], pl["slot_expert"], pl["n_slots"])
        if l == 0:                       # same inputs on both sides here: the product itself, row by row
            assert_close(to_host(y_on), y, synth.BF16, "layer 0 y_perm")
            _assert_rows_close(to_host(y_on), y, "layer 0 y_perm")
        ref_x = oracle.combine(y, ref_x, dp["inv"], g_prob, 1)
        assert_close(to_host(nxt), ref_x, synth.BF16, f"layer {l} out")
        cur, nxt = nxt, cur
        del w1, w2, w1h, w2h
        print(f"workload 5 layer {l}: slots {pl['n_slots']}, hot expert {n.max()} tokens in "
              f"{pl['replicas'].max()} slots, {flips} near-tie flips, t={time.time() - t0:.1f}s", flush=True)
    assert most_slots >= 32             # ceil(32768 / 1024) slots for the hot expert
