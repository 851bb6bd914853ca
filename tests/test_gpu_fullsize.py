"""Full-size GPU parity on the large workloads, in the launch configuration bench.py times.

The oracle cannot evaluate these sizes whole in test time, so: integer stages (plan, dispatch)
are compared bit for bit at full size against the oracle fed the GPU's own router ids; float
stages are compared on sampled rows / tokens that the oracle evaluates one by one; and
size-independent properties (conservation, no drops, passthrough) are checked on everything.
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
    # sampled rows: include the first and last rows of the hottest expert and the global tail
    rng = np.random.default_rng(4)
    hot = int(np.argmax(dp["kept"]))
    rows = np.unique(np.concatenate([rng.choice(K, 80, replace=False), [0, K - 1, dp["expert_offset"][hot],
                                     dp["expert_offset"][hot + 1] - 1]])).astype(np.int32)
    xp = np.zeros_like(c["x"])
    xp[rows] = c["x"][dp["perm"][rows]]
    y = oracle.ffn(xp, c["w1"], c["w2"], dp["slot_offset"], pl["slot_expert"], pl["n_slots"], rows=rows)
    assert_close(to_host(layer.y_perm)[rows], y[rows], synth.BF16, "y_perm sample")
    ref_out = oracle.combine(y, c["x"], dp["inv"], g_prob, 0)
    toks = dp["perm"][rows]
    assert_close(got[toks], ref_out[toks], synth.BF16, "out sample")
    # replication off (same plan): identical outputs
    out_off = layer.forward(x, wr, b, w1, w2, schedule=moe.SCHEDULE_EXPERTS, router_layout=moe.LAYOUT_PACKED)
    assert torch.equal(out, out_off)
    print(f"workload 4 C={C}: kept {K}/{T}, slots {pl['n_slots']}, {flips} near-tie flips, "
          f"total {time.time() - t0:.1f}s", flush=True)


@pytest.mark.timeout(900)
def test_workload5_stack_full_size():
    """6-layer stack, T=65536, E=256, one expert at 50% load, nothing may drop.  Sampled tokens
    are followed through all six layers by the oracle alone (with no drops a token's result
    depends on the other tokens only through ranks)."""
    import paper_2605_11537_amd as moe
    t0 = time.time()
    c = synth.config_inputs(5, weights=False)
    T, d, F, E, R, C, NL = c["T"], c["d"], c["F"], c["E"], c["R"], c["C"], c["n_layers"]
    seed = synth.workloads.SEED0 + 5
    layer = moe.MoeLayer(T, d, F, E, R, C, torch.bfloat16)
    rng = np.random.default_rng(5)
    sample = np.sort(rng.choice(T, 24, replace=False))
    ref_x = c["x"][sample].copy()                      # oracle-side state of the sampled tokens
    cur = to_dev(c["x"])
    nxt = torch.empty_like(cur)
    hot_rows_seen = 0
    for l in range(NL):
        lay = c["layers"][l]
        w1h = synth.normal_tensor((E, d, F), 0.02, [seed, 50 + l], synth.BF16)
        w2h = synth.normal_tensor((E, F, d), 0.02, [seed, 60 + l], synth.BF16)
        w1, w2 = moe.moe_pack_weights(to_dev(w1h)), moe.moe_pack_weights(to_dev(w2h))
        wr = to_dev(lay["w_router"])
        layer.forward(cur, wr, None, w1, w2, residual=1, out=nxt)
        torch.cuda.synchronize()
        g_idx, g_prob = to_host(layer.route_out[0]), to_host(layer.route_out[1])
        pl, dp = _integer_parity(moe, layer, g_idx, E, C, R, T)
        assert int(dp["expert_offset"][E]) == T and (dp["inv"] >= 0).all()      # nothing drops
        n = dp["counts"]
        assert n.max() >= 0.49 * T                                              # the hot expert
        hot_rows_seen = max(hot_rows_seen, int(pl["replicas"].max()))
        # sampled tokens, one by one, from the oracle's own previous-layer state
        rt = oracle.route(ref_x, lay["w_router"], None)
        tau = 1e-4 * max(1.0, np.abs(rt["logits"]).max())
        check_ids_margin(g_idx[sample], rt["idx"], rt["idx2"], rt["margin"], tau, f"layer {l} route")
        new_ref = np.empty_like(ref_x)
        for i in range(sample.size):
            e = int(g_idx[sample[i]])
            y = oracle.ffn(ref_x[i:i + 1], w1h, w2h, np.array([0, 1], np.int32), np.array([e], np.int32), 1)
            new_ref[i] = oracle.combine(y, ref_x[i:i + 1], np.array([0], np.int32),
                                        g_prob[sample[i]:sample[i] + 1], 1)[0]
        ref_x = new_ref
        got = to_host(nxt[torch.from_numpy(sample).cuda()])
        assert_close(got, ref_x, synth.BF16, f"layer {l} sampled tokens")
        cur, nxt = nxt, cur
        del w1, w2, w1h, w2h
        print(f"workload 5 layer {l}: slots {pl['n_slots']}, hot expert {n.max()} tokens in "
              f"{pl['replicas'].max()} slots, t={time.time() - t0:.1f}s", flush=True)
    assert hot_rows_seen >= 32          # ceil(32768 / 1024) slots for the hot expert
