"""moe_plan_dispatch on the GPU: the one-call form of replica_plan + the index tables of moe_dispatch.
Its tables are held bit for bit against the oracle and against the two separate calls, for sizes that
take the single-kernel path, sizes at its limits, and sizes that fall back to the separate kernels."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import to_dev, to_host

pytestmark = pytest.mark.gpu


def _ids(n, E, s, seed):
    rng = np.random.default_rng(seed)
    return rng.choice(E, size=n, p=synth.zipf_weights(E, s)).astype(np.int32)


@pytest.mark.parametrize("T,n_plan,E,R,C,policy", [
    (4096, 4096, 128, 16, 40, 0),       # the Switch-base-128 workload's sizes
    (4096, 4096, 128, 16, 40, 1),
    (1000, 777, 24, 5, 30, 0),          # ragged, plan ids of another length
    (8192, 8192, 256, 32, 20, 0),       # the limits of the single-kernel path
    (1, 1, 4, 2, 1, 0),
    (0, 0, 8, 2, 4, 0),                 # empty batch: tables only
    (300, 300, 8, 0, 20, 0),            # no budget
    (20000, 20000, 64, 9, 200, 0),      # falls back to the separate kernels
    (5000, 9000, 300, 12, 10, 1),       # E above the single-kernel limit
])
def test_plan_dispatch_equals_oracle_and_separate_calls(T, n_plan, E, R, C, policy):
    import paper_2605_11537_amd as moe
    ids = _ids(T, E, 1.1, 7 + T)
    pids = ids if n_plan == T and T % 2 == 0 else _ids(n_plan, E, 1.3, 8 + n_plan)
    pl = oracle.plan(pids, E, R, C, policy)
    dp = oracle.dispatch(np.zeros((T, 4), np.float32), ids, pl["replicas"], E, C, E + R)
    dev_ids = to_dev(ids) if T else torch.empty(0, dtype=torch.int32, device="cuda")
    dev_pids = to_dev(pids) if n_plan else torch.empty(0, dtype=torch.int32, device="cuda")
    if pids is ids:
        dev_pids = dev_ids            # the plan made from the routed ids themselves: one buffer for both
    gp, gd = moe.moe_plan_dispatch(dev_pids, dev_ids, E, R, C, policy)
    for name, rk in (("plan_counts", "counts"), ("replicas", "replicas"), ("slot_base", "slot_base"),
                     ("slot_expert", "slot_expert")):
        assert (to_host(gp[name]) == pl[rk]).all(), name
    assert int(gp["n_slots"].item()) == pl["n_slots"]
    for name in ("counts", "kept", "expert_offset", "slot_offset", "perm", "inv"):
        assert (to_host(gd[name]) == dp[name]).all(), name
    if T:
        sp = moe.replica_plan(dev_pids, E, R, C, policy)
        sd = moe.moe_dispatch(None, dev_ids, sp["replicas"], E, C, E + R, shape=(T, 8), dtype=torch.bfloat16)
        for name in gp:
            assert torch.equal(gp[name], sp[name]), name
        for name in ("counts", "kept", "expert_offset", "slot_offset", "perm", "inv"):
            assert torch.equal(gd[name], sd[name]), name
        if pids is ids:
            # the same ids from a second buffer take the other build of the kernel: same tables
            gp2, gd2 = moe.moe_plan_dispatch(dev_ids.clone(), dev_ids, E, R, C, policy)
            for name in gp:
                assert torch.equal(gp[name], gp2[name]), name
            for name in ("kept", "slot_offset", "perm", "inv"):
                assert torch.equal(gd[name], gd2[name]), name


@pytest.mark.parametrize("T,k,E,R,C", [(1000, 3, 16, 6, 150), (2730, 3, 128, 16, 70), (4000, 3, 32, 4, 300)])
def test_plan_dispatch_topk(T, k, E, R, C):
    """[k,T] ids: the assignments of a top-k layer (the last case is above the single-kernel limit)."""
    import paper_2605_11537_amd as moe
    rng = np.random.default_rng(T)
    score = np.log(synth.zipf_weights(E, 1.1))[None, :] + rng.gumbel(size=(T, E))
    ids = np.ascontiguousarray(np.argsort(-score, axis=1)[:, :k].T.astype(np.int32))
    gp, gd = moe.moe_plan_dispatch(to_dev(ids.reshape(-1)), to_dev(ids), E, R, C)
    sp = moe.replica_plan(to_dev(ids.reshape(-1)), E, R, C)
    sd = moe.moe_dispatch_topk(None, to_dev(ids), sp["replicas"], E, C, E + R, shape=(T, 8), dtype=torch.bfloat16)
    for name in gp:
        assert torch.equal(gp[name], sp[name]), name
    for name in ("counts", "kept", "expert_offset", "slot_offset", "perm", "inv", "row_token"):
        assert torch.equal(gd[name], sd[name]), name
    pl = oracle.plan(ids.reshape(-1), E, R, C)
    dp = oracle.dispatch(np.zeros((k * T, 4), np.float32), ids.reshape(-1), pl["replicas"], E, C, E + R)
    assert (to_host(gd["perm"]) == dp["perm"]).all() and (to_host(gd["inv"]).reshape(-1) == dp["inv"]).all()
    assert (to_host(gd["row_token"]) == np.where(dp["perm"] >= 0, dp["perm"] % T, -1)).all()
    assert (dp["inv"] < 0).any()


def test_plan_dispatch_repeated_calls_reuse_buffers():
    """Second call with other ids into the same output buffers: nothing of the first call survives."""
    import paper_2605_11537_amd as moe
    E, R, C, T = 64, 8, 50, 3000
    a, b = _ids(T, E, 1.2, 1), _ids(T, E, 0.3, 2)
    gp, gd = moe.moe_plan_dispatch(to_dev(a), to_dev(a), E, R, C)
    moe.moe_plan_dispatch(to_dev(b), to_dev(b), E, R, C, plan_out=gp, disp_out=gd)
    pl = oracle.plan(b, E, R, C)
    dp = oracle.dispatch(np.zeros((T, 4), np.float32), b, pl["replicas"], E, C, E + R)
    assert (to_host(gp["slot_expert"]) == pl["slot_expert"]).all()
    for name in ("kept", "slot_offset", "perm", "inv"):
        assert (to_host(gd[name]) == dp[name]).all(), name


def test_layer_forward_replays_from_a_hip_graph():
    """The whole layer is a fixed sequence of launches on preallocated buffers (no allocation, no memset,
    no synchronisation inside the library), so it can be captured once and replayed.  Every replay, with
    new token values in the captured input buffer and eager work in between, equals the eager result."""
    import paper_2605_11537_amd as moe
    T, d, F, E, R, C = 2000, 128, 256, 16, 6, 150
    c = synth.moe_layer_inputs(T, d, F, E, synth.BF16, 1.2, 555)
    layer = moe.MoeLayer(T, d, F, E, R, C, torch.bfloat16)
    eager = moe.MoeLayer(T, d, F, E, R, C, torch.bfloat16)
    wr, b = to_dev(c["w_router"]), to_dev(c["b_router"])
    w1, w2 = moe.moe_pack_weights(to_dev(c["w1"])), moe.moe_pack_weights(to_dev(c["w2"]))
    x_static = to_dev(c["x"]).clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(2):
            layer.forward(x_static, wr, b, w1, w2, residual=1)       # warm up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        out_static = layer.forward(x_static, wr, b, w1, w2, residual=1)
    plans = set()
    for i in range(4):
        x_new = synth.normal_tensor((T, d), 1.0 + 0.5 * i, [556, i], synth.BF16)
        x_static.copy_(to_dev(x_new))
        graph.replay()
        torch.cuda.synchronize()
        got = out_static.clone()
        want = eager.forward(to_dev(x_new), wr, b, w1, w2, residual=1)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"replay {i}"
        assert torch.equal(layer.disp_out["inv"], eager.disp_out["inv"])
        plans.add(tuple(to_host(layer.plan_out["replicas"]).tolist()))
    assert len(plans) > 1                                            # the replays really planned anew
