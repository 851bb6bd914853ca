"""GPU parity: every C-ABI call against the CPU oracle on the same seeded inputs.

Integer work (plan, histogram, offsets, permutation, slot tables) must match bit for bit.
Float outputs: fp32 max abs error 1e-4, bf16 max relative error 2e-2.  Float->int decisions
(router and predictor argmax) must equal the oracle's wherever its top-2 gap exceeds the
binary32 accumulation noise, and be the runner-up otherwise; stages downstream of such a
decision are compared with the oracle re-run on the GPU's own ids.
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import assert_close, check_ids_margin, f64, to_dev, to_host

pytestmark = pytest.mark.gpu

moe = None


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global moe
    import paper_2605_11537_amd as m
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    m.lib()
    moe = m
    yield


def _sync():
    torch.cuda.synchronize()


# --------------------------------------------------------------------------- replica_plan
@pytest.mark.parametrize("policy", [0, 1])
def test_plan_bit_exact_random(policy):
    rng = np.random.default_rng(40 + policy)
    cases = [(0, 4, 3, 2), (1, 1, 0, 1), (700, 8, 4, 80), (4096, 128, 16, 40), (5000, 100, 37, 7),
             (16384, 256, 32, 64), (3000, 1024, 100, 2), (2048, 64, 4000, 1), (777, 3, 0, 5),
             (8193, 7, 3, 300), (70001, 300, 64, 128)]
    for T, E, R, C in cases:
        p = rng.dirichlet(np.ones(E) * 0.2)
        ids = rng.choice(E, size=T, p=p).astype(np.int32)
        ref = oracle.plan(ids, E, R, C, policy)
        got = moe.replica_plan(to_dev(ids) if T else torch.empty(0, dtype=torch.int32, device="cuda"),
                               E, R, C, policy)
        _sync()
        print(f"plan T={T} E={E} R={R} C={C} policy={policy}", flush=True)
        assert (to_host(got["plan_counts"]) == ref["counts"]).all()
        assert (to_host(got["replicas"]) == ref["replicas"]).all()
        assert (to_host(got["slot_base"]) == ref["slot_base"]).all()
        assert (to_host(got["slot_expert"]) == ref["slot_expert"]).all()
        assert int(got["n_slots"].item()) == ref["n_slots"]


@pytest.mark.parametrize("policy", [0, 1])
def test_plan_hand_out_ties_and_long_tail(policy):
    """Cases made for the slot-by-slot hand-out after the floors: many experts with equal load per slot
    (the lower id must win every tie), a budget far below the wants, and wants met one slot at a time."""
    cases = []
    E, C = 128, 10
    counts = np.full(E, 25)                     # all equal: 2 extra slots wanted each, 37 to hand out
    cases.append((counts, 37, C))
    counts = np.array([100 - (i % 7) for i in range(300)])   # blocks of equal loads, R below the wants
    cases.append((counts, 64, 9))
    counts = np.array([1000, 999, 501, 500, 250, 3, 2, 1, 0, 0])
    cases.append((counts, 13, 17))
    counts = np.array([60, 40, 40, 20, 20, 20] * 20)          # equal fractions n/r across different n and r
    cases.append((counts, 50, 10))
    rng = np.random.default_rng(77)
    for counts, R, C in cases:
        E = len(counts)
        ids = np.repeat(np.arange(E), counts).astype(np.int32)
        rng.shuffle(ids)
        ref = oracle.plan(ids, E, R, C, policy)
        got = moe.replica_plan(to_dev(ids), E, R, C, policy)
        assert (to_host(got["replicas"]) == ref["replicas"]).all(), (E, R, C)
        assert (to_host(got["slot_expert"]) == ref["slot_expert"]).all()
        assert ref["replicas"].sum() == E + R                  # the budget binds in every case
        if len(ids) <= 8192 and E <= 256:
            gp, _ = moe.moe_plan_dispatch(to_dev(ids), to_dev(ids[::-1].copy()), E, R, C, policy)
            assert (to_host(gp["replicas"]) == ref["replicas"]).all()


@pytest.mark.timeout(300)
def test_plan_above_2_pow_24_ids():
    """More than 2^24 ids: counts beyond the range of the packed hand-out keys (the binary64 keys run)."""
    T, E, R, C = (1 << 24) + 12345, 64, 20, 150000
    rng = np.random.default_rng(5)
    ids = rng.choice(E, size=T, p=synth.zipf_weights(E, 0.9)).astype(np.int32)
    ref = oracle.plan(ids, E, R, C)
    got = moe.replica_plan(to_dev(ids), E, R, C)
    assert (to_host(got["plan_counts"]) == ref["counts"]).all()
    assert (to_host(got["replicas"]) == ref["replicas"]).all()
    assert ref["counts"].max() >= (1 << 21) and ref["replicas"].sum() == E + R


def test_plan_paper_scenario_on_gpu():
    ids = np.array([5] * 32 + [9] * 32, np.int32)
    np.random.default_rng(0).shuffle(ids)
    got = moe.replica_plan(to_dev(ids), 64, 62, 1)
    r = to_host(got["replicas"])
    assert r[5] == 32 and r[9] == 32 and r.sum() == 64 + 62


# --------------------------------------------------------------------------- moe_dispatch
DISPATCH_CASES = [
    # T, d, E, C, R, dtype
    (1, 8, 1, 1, 0, synth.F32),
    (63, 8, 3, 5, 2, synth.F32),
    (512, 64, 8, 80, 4, synth.F32),
    (1024, 16, 8, 100, 3, synth.BF16),
    (1025, 16, 8, 100, 3, synth.BF16),
    (4096, 768, 128, 40, 16, synth.BF16),
    (5000, 72, 100, 9, 20, synth.BF16),
    (3001, 8, 1024, 2, 50, synth.BF16),
    (16384, 128, 256, 64, 32, synth.BF16),
    (70001, 32, 300, 150, 64, synth.BF16),
]


@pytest.mark.parametrize("T,d,E,C,R,dtype", DISPATCH_CASES)
def test_dispatch_bit_exact(T, d, E, C, R, dtype):
    rng = np.random.default_rng(T * 7 + E)
    ids = rng.choice(E, size=T, p=rng.dirichlet(np.ones(E) * 0.3)).astype(np.int32)
    x = synth.normal_tensor((T, d), 1.0, [T, E, 1], dtype)
    rep = oracle.plan(ids, E, R, C)["replicas"]
    for replicas in (rep, None):
        ref = oracle.dispatch(x, ids, replicas, E, C, E + R)
        got = moe.moe_dispatch(to_dev(x), to_dev(ids), to_dev(replicas), E, C, E + R)
        _sync()
        K = int(ref["expert_offset"][E])
        for k in ("counts", "kept", "expert_offset", "slot_offset", "perm", "inv"):
            assert (to_host(got[k]) == ref[k]).all(), k
        assert (to_host(got["x_perm"])[:K] == ref["x_perm"][:K]).all()


def test_dispatch_is_deterministic():
    rng = np.random.default_rng(3)
    T, E = 8192, 256
    ids = to_dev(rng.choice(E, size=T, p=rng.dirichlet(np.ones(E) * 0.1)).astype(np.int32))
    x = to_dev(synth.normal_tensor((T, 64), 1.0, [9], synth.BF16))
    first = moe.moe_dispatch(x, ids, None, E, 48, E)
    for _ in range(10):
        again = moe.moe_dispatch(x, ids, None, E, 48, E)
        assert torch.equal(first["perm"], again["perm"]) and torch.equal(first["inv"], again["inv"])


# --------------------------------------------------------------------------- moe_combine
@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
@pytest.mark.parametrize("residual", [0, 1])
def test_combine(dtype, residual):
    rng = np.random.default_rng(8)
    T, d = 1000, 72 if dtype == synth.BF16 else 68
    x = synth.normal_tensor((T, d), 1.0, [1], dtype)
    y = synth.normal_tensor((T, d), 0.5, [2], dtype)
    perm = rng.permutation(T)[:700]
    inv = np.full(T, -1, np.int32)
    inv[perm] = np.arange(700)
    p = rng.random(T).astype(np.float32)
    ref = oracle.combine(y, x, inv, p, residual)
    got = to_host(moe.moe_combine(to_dev(y), to_dev(x), to_dev(inv), to_dev(p), residual))
    assert (got[inv < 0] == x[inv < 0]).all()                 # passthrough: bit identical
    assert_close(got, ref, dtype, "combine")
    if dtype == synth.BF16:
        assert (got == ref).mean() > 0.999                    # one rounding on both sides
    else:
        assert np.abs(f64(got) - f64(ref)).max() <= 1e-6


# --------------------------------------------------------------------------- moe_route
def test_route_config1_identical():
    c = synth.config_inputs(1, weights=False)
    ref = oracle.route(c["x"], c["w_router"], c["b_router"])
    idx, prob, logits = moe.moe_route(to_dev(c["x"]), to_dev(c["w_router"]), to_dev(c["b_router"]), want_logits=True)
    assert (to_host(idx) == ref["idx"]).all()
    assert np.abs(to_host(prob) - ref["prob"]).max() <= 1e-6
    assert np.abs(to_host(logits) - ref["logits"]).max() <= 1e-5


@pytest.mark.parametrize("T,d,E,bias", [(4096, 768, 128, True), (1000, 768, 256, True), (333, 128, 128, False),
                                        (500, 64, 24, True), (70, 256, 512, False),
                                        # 256 experts from 16384 tokens on: persistent workgroups, router matrix in
                                        # registers; more tiles than workgroups, a ragged last tile, every width built
                                        (16384 + 21, 768, 256, True), (16385, 512, 256, False), (40000, 256, 256, True)])
def test_route_bf16(T, d, E, bias):
    c = synth.moe_layer_inputs(T, d, 8, E, synth.BF16, 1.0, 900 + T, weights=False)
    b = c["b_router"] if bias else None
    ref = oracle.route(c["x"], c["w_router"], b)
    idx, prob, logits = moe.moe_route(to_dev(c["x"]), to_dev(c["w_router"]), to_dev(b), want_logits=True)
    lg = to_host(logits)
    assert np.abs(lg - ref["logits"]).max() <= 1e-4 * max(1.0, np.abs(ref["logits"]).max())
    tau = 1e-4 * max(1.0, np.abs(ref["logits"]).max())
    flips = check_ids_margin(to_host(idx), ref["idx"], ref["idx2"], ref["margin"], tau, "route")
    same = to_host(idx) == ref["idx"]
    assert np.abs(to_host(prob) - ref["prob"])[same].max() <= 1e-4
    print(f"route T={T} E={E}: {flips} near-tie flips", flush=True)
    if E in (128, 256) and d % 128 == 0:
        # router matrix packed once by the caller: same kernel, same bits
        wp = moe.moe_pack_weights(to_dev(c["w_router"])[None].contiguous())[0]
        idx2, prob2, _ = moe.moe_route(to_dev(c["x"]), wp, to_dev(b), w_layout=moe.LAYOUT_PACKED)
        assert torch.equal(idx, idx2) and torch.equal(prob, prob2)


# --------------------------------------------------------------------------- pack + expert FFN
def test_pack_weights_layout_bit_exact():
    E, K, N = 3, 64, 160
    w = synth.normal_tensor((E, K, N), 1.0, [5], synth.BF16)
    got = to_host(moe.moe_pack_weights(to_dev(w)))
    # [e][n/32][k/8][n%32][k%8]
    ref = w.reshape(E, K // 8, 8, N // 32, 32).transpose(0, 3, 1, 4, 2)
    assert (got.reshape(-1) == ref.reshape(-1)).all()


def _slots_for(rows_per_slot, experts):
    so = np.concatenate([[0], np.cumsum(rows_per_slot)]).astype(np.int32)
    return so, np.asarray(experts, np.int32)


@pytest.mark.parametrize("schedule", [0, 1])
def test_ffn_fp32_config1(schedule):
    c = synth.config_inputs(1)
    L = oracle.layer(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"], c["C"], c["R"])
    dp, pl = L["dispatch"], L["plan"]
    y = moe.moe_expert_ffn(to_dev(dp["x_perm"]), to_dev(c["w1"]), to_dev(c["w2"]), to_dev(dp["slot_offset"]),
                           to_dev(pl["slot_expert"]), torch.tensor([pl["n_slots"]], dtype=torch.int32, device="cuda"),
                           c["E"], c["F"], schedule=schedule)
    K = int(dp["expert_offset"][c["E"]])
    assert_close(to_host(y)[:K], L["y_perm"][:K], synth.F32, "ffn fp32")


@pytest.mark.parametrize("schedule", [0, 1])
def test_ffn_bf16_ragged_slots(schedule):
    E, d, F = 5, 128, 256
    rows = [3, 0, 64, 65, 1, 130, 40, 0, 17]
    experts = [0, 0, 1, 2, 2, 3, 3, 3, 4]
    so, se = _slots_for(rows, experts)
    T = int(so[-1]) + 11                        # rows past the last slot stay untouched
    x = synth.normal_tensor((T, d), 1.0, [11], synth.BF16)
    w1 = synth.normal_tensor((E, d, F), 0.05, [12], synth.BF16)
    w2 = synth.normal_tensor((E, F, d), 0.05, [13], synth.BF16)
    ref = oracle.ffn(x, w1, w2, so, se, len(rows))
    so_pad = np.concatenate([so, np.full(4, so[-1], np.int32)])
    se_pad = np.concatenate([se, np.full(4, -1, np.int32)])
    sentinel = torch.full((T, d), 7.0, dtype=torch.bfloat16, device="cuda")
    y = moe.moe_expert_ffn(to_dev(x), moe.moe_pack_weights(to_dev(w1)), moe.moe_pack_weights(to_dev(w2)),
                           to_dev(so_pad), to_dev(se_pad), torch.tensor([len(rows)], dtype=torch.int32, device="cuda"),
                           E, F, schedule=schedule, out=sentinel)
    got = to_host(y)
    K = int(so[-1])
    assert_close(got[:K], ref[:K], synth.BF16, "ffn bf16")
    assert (f64(got[K:]) == 7.0).all()
    # element-wise: bf16 storage of y allows half an ulp of each value plus accumulation noise
    g, r = f64(got[:K]), f64(ref[:K])
    assert (np.abs(g - r) <= 2.0 ** -7 * np.abs(r) + 1e-3 * np.abs(r).max()).all()


@pytest.mark.parametrize("schedule", [0, 1])
def test_ffn_bf16_long_slots(schedule):
    """Few long slots spanning many row tiles; ragged row counts around the tile height, an
    empty slot, and the fused gather."""
    E, d, F = 3, 256, 512
    rows = [300, 129, 0, 128, 1, 700]
    experts = [0, 0, 1, 1, 2, 2]
    so, se = _slots_for(rows, experts)
    K = int(so[-1])
    T = K + 5
    x = synth.normal_tensor((T, d), 1.0, [21], synth.BF16)
    w1 = synth.normal_tensor((E, d, F), 0.05, [22], synth.BF16)
    w2 = synth.normal_tensor((E, F, d), 0.05, [23], synth.BF16)
    ref = oracle.ffn(x, w1, w2, so, se, len(rows))
    args = (moe.moe_pack_weights(to_dev(w1)), moe.moe_pack_weights(to_dev(w2)), to_dev(so), to_dev(se),
            torch.tensor([len(rows)], dtype=torch.int32, device="cuda"), E, F)
    y = moe.moe_expert_ffn(to_dev(x), *args, schedule=schedule)
    assert_close(to_host(y)[:K], ref[:K], synth.BF16, "ffn bf16 large tiles")
    g, r = f64(to_host(y)[:K]), f64(ref[:K])
    assert (np.abs(g - r) <= 2.0 ** -7 * np.abs(r) + 1e-3 * np.abs(r).max()).all()
    # fused gather: rows arrive through an index
    perm = np.random.default_rng(1).permutation(T).astype(np.int32)
    x_src = np.zeros_like(x)
    x_src[perm] = x
    y2 = moe.moe_expert_ffn(to_dev(x_src), *args, schedule=schedule, row_index=to_dev(perm))
    assert torch.equal(y[:K], y2[:K])


@pytest.mark.parametrize("case", ["ragged", "long", "dense"])
def test_ffn_first_product_h(case):
    """The first product on its own: h = relu(x_perm W1[e]) as left in the head of the workspace, element by
    element against the oracle, for the three kernels that can write it (64/128-row tiles of the 128-column
    kernel reading the slot tables, the same with a work list, the 256 x 256 tile kernel)."""
    if case == "ragged":
        E, d, F = 5, 128, 256
        rows, experts = [3, 0, 64, 65, 1, 130, 40, 0, 17], [0, 0, 1, 2, 2, 3, 3, 3, 4]
    elif case == "long":
        E, d, F = 3, 256, 512
        rows, experts = [300, 129, 0, 128, 1, 700], [0, 0, 1, 1, 2, 2]
    else:
        E, d, F = 4, 256, 512
        rows, experts = [1500, 129, 0, 256, 257, 1, 385, 2000, 63], [0, 0, 1, 1, 2, 2, 3, 3, 3]
    so, se = _slots_for(rows, experts)
    K = int(so[-1])
    T = K + 9
    x = synth.normal_tensor((T, d), 1.0, [51], synth.BF16)
    w1 = synth.normal_tensor((E, d, F), 0.05, [52], synth.BF16)
    w2 = synth.normal_tensor((E, F, d), 0.05, [53], synth.BF16)
    ref_y, ref_h = oracle.ffn(x, w1, w2, so, se, len(rows), want_h=True)
    ws = torch.zeros(moe.lib().moe_expert_ffn_workspace_bytes(T, len(rows), d, F, moe.MOE_BF16), dtype=torch.uint8,
                     device="cuda")
    y = moe.moe_expert_ffn(to_dev(x), moe.moe_pack_weights(to_dev(w1)), moe.moe_pack_weights(to_dev(w2)),
                           to_dev(so), to_dev(se), torch.tensor([len(rows)], dtype=torch.int32, device="cuda"),
                           E, F, ws=ws)
    _sync()
    h = to_host(ws[:T * F * 2].view(torch.bfloat16).view(T, F))
    assert (f64(ref_h[:K]) > 0).mean() > 0.3 and (f64(ref_h[:K]) == 0).mean() > 0.3    # the ReLU cuts about half
    assert_close(h[:K], ref_h[:K], synth.BF16, "h")
    g, r = f64(h[:K]), f64(ref_h[:K])
    assert (np.abs(g - r) <= 2.0 ** -7 * np.abs(r) + 1e-3 * np.abs(r).max()).all()
    assert ((g == 0) == (r == 0)).mean() > 0.999           # zeros of the ReLU in the same places (up to rounding at 0)
    assert (h[K:] == 0).all()                              # rows outside all slots are not written
    assert_close(to_host(y)[:K], ref_y[:K], synth.BF16, "y")


def test_ffn_timed_call_equals_untimed_and_records_its_events():
    """moe_expert_ffn_timed (measurement section of the header): same bits as moe_expert_ffn, three events
    recorded in order around the two products."""
    E, d, F = 4, 128, 256
    rows, experts = [70, 3, 0, 129, 64], [0, 1, 1, 2, 3]
    so, se = _slots_for(rows, experts)
    T = int(so[-1])
    x = to_dev(synth.normal_tensor((T, d), 1.0, [61], synth.BF16))
    w1 = moe.moe_pack_weights(to_dev(synth.normal_tensor((E, d, F), 0.05, [62], synth.BF16)))
    w2 = moe.moe_pack_weights(to_dev(synth.normal_tensor((E, F, d), 0.05, [63], synth.BF16)))
    args = (w1, w2, to_dev(so), to_dev(se), torch.tensor([len(rows)], dtype=torch.int32, device="cuda"), E, F)
    y = moe.moe_expert_ffn(x, *args)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for e in evs:
        e.record()
    y_t = moe.moe_expert_ffn(x, *args, events=evs)
    _sync()
    assert torch.equal(y, y_t)
    assert evs[0].elapsed_time(evs[1]) > 0 and evs[1].elapsed_time(evs[2]) > 0


def test_ffn_bf16_dense_tiles():
    """Enough rows that the 256 x 256 tile kernel takes the slots: lengths around its cut points
    (pieces of 1..256 rows use 1..8 row blocks of the tile), short and empty slots beside them, and
    the fused gather."""
    E, d, F = 7, 256, 512
    rows = [1500, 129, 0, 256, 257, 1, 385, 2000, 128, 513, 384, 64, 65, 96, 289, 320, 321, 32, 160, 224, 97]
    experts = [0, 0, 1, 1, 2, 2, 3, 3, 3, 4, 4, 4, 5, 5, 5, 5, 6, 6, 6, 6, 6]
    so, se = _slots_for(rows, experts)
    K = int(so[-1])
    T = K + 3
    assert T >= 4096 and T >= 64 * len(rows)        # the sizes at which the library uses that kernel
    x = synth.normal_tensor((T, d), 1.0, [31], synth.BF16)
    w1 = synth.normal_tensor((E, d, F), 0.05, [32], synth.BF16)
    w2 = synth.normal_tensor((E, F, d), 0.05, [33], synth.BF16)
    ref = oracle.ffn(x, w1, w2, so, se, len(rows))
    args = (moe.moe_pack_weights(to_dev(w1)), moe.moe_pack_weights(to_dev(w2)), to_dev(so), to_dev(se),
            torch.tensor([len(rows)], dtype=torch.int32, device="cuda"), E, F)
    y = moe.moe_expert_ffn(to_dev(x), *args)
    _sync()
    assert_close(to_host(y)[:K], ref[:K], synth.BF16, "ffn bf16 dense tiles")
    g, r = f64(to_host(y)[:K]), f64(ref[:K])
    assert (np.abs(g - r) <= 2.0 ** -7 * np.abs(r) + 1e-3 * np.abs(r).max()).all()
    # replication off walks whole experts with the 128-column kernel only: same sums in the same order
    y_off = moe.moe_expert_ffn(to_dev(x), *args, schedule=1)
    assert torch.equal(y[:K], y_off[:K])
    perm = np.random.default_rng(2).permutation(T).astype(np.int32)
    x_src = np.zeros_like(x)
    x_src[perm] = x
    y2 = moe.moe_expert_ffn(to_dev(x_src), *args, row_index=to_dev(perm))
    assert torch.equal(y[:K], y2[:K])
    y3 = moe.moe_expert_ffn(to_dev(x), *args)           # twice in a row: nothing stale in the work lists
    assert torch.equal(y, y3) or torch.equal(y[:K], y3[:K])


def test_ffn_bf16_many_short_slots_beside_long_ones():
    """The tile kernel on matrices other than the small test's (d = 512, F = 768: two and three column tiles,
    16 and 24 k stages): rests of 1..128 rows with 1..4 row blocks beside full 256-row ranges and rests above
    128 rows, 32 single-slot experts of 1..128 rows (tiles that only stream their weights), an expert with two
    short slots (shared weights), empty slots, the fused gather.  Every element of h and of the output against
    the oracle, and bit for bit against the experts schedule, which runs the 128-column kernel alone and
    accumulates in the same order."""
    E, d, F = 40, 512, 768
    rng = np.random.default_rng(7)
    rows = [1500, 129, 0, 256, 257, 1, 385, 2000, 128, 513, 384, 64, 65, 96, 289, 320, 321, 32, 160, 224, 97, 127, 33]
    experts = [0, 0, 1, 1, 2, 2, 3, 3, 3, 4, 4, 4, 5, 5, 5, 5, 6, 6, 6, 6, 6, 7, 7]
    for e in range(8, E):                         # many single-slot experts with short rows
        rows.append(int(rng.integers(1, 129)))
        experts.append(e)
    so, se = _slots_for(rows, experts)
    K = int(so[-1])
    T = K + 5
    assert T >= 4096 and T >= 64 * len(rows)        # the sizes at which the library uses the tile kernels
    x = synth.normal_tensor((T, d), 1.0, [71], synth.BF16)
    w1 = synth.normal_tensor((E, d, F), 0.05, [72], synth.BF16)
    w2 = synth.normal_tensor((E, F, d), 0.05, [73], synth.BF16)
    ref_y, ref_h = oracle.ffn(x, w1, w2, so, se, len(rows), want_h=True)
    args = (moe.moe_pack_weights(to_dev(w1)), moe.moe_pack_weights(to_dev(w2)), to_dev(so), to_dev(se),
            torch.tensor([len(rows)], dtype=torch.int32, device="cuda"), E, F)
    ws = torch.zeros(moe.lib().moe_expert_ffn_workspace_bytes(T, len(rows), d, F, moe.MOE_BF16), dtype=torch.uint8,
                     device="cuda")
    y = moe.moe_expert_ffn(to_dev(x), *args, ws=ws)
    _sync()
    h = to_host(ws[:T * F * 2].view(torch.bfloat16).view(T, F))
    assert_close(h[:K], ref_h[:K], synth.BF16, "h, many short slots")
    assert (h[K:] == 0).all()                       # rows outside all slots are not written
    assert_close(to_host(y)[:K], ref_y[:K], synth.BF16, "ffn bf16, many short slots")
    g, r = f64(to_host(y)[:K]), f64(ref_y[:K])
    assert (np.abs(g - r) <= 2.0 ** -7 * np.abs(r) + 1e-3 * np.abs(r).max()).all()
    y_off = moe.moe_expert_ffn(to_dev(x), *args, schedule=1)
    assert torch.equal(y[:K], y_off[:K])
    perm = np.random.default_rng(2).permutation(T).astype(np.int32)
    x_src = np.zeros_like(x)
    x_src[perm] = x
    y2 = moe.moe_expert_ffn(to_dev(x_src), *args, row_index=to_dev(perm))
    assert torch.equal(y[:K], y2[:K])
    y3 = moe.moe_expert_ffn(to_dev(x), *args)           # twice in a row: nothing stale in the work lists
    assert torch.equal(y[:K], y3[:K])


def test_ffn_bf16_short_tiles_several_per_workgroup():
    """More short row ranges x column tiles than the chip has compute units: every persistent workgroup of the
    tile kernel walks several tiles of at most 128 rows (loads of the next tile's first stages and its row
    numbers issued during the current one, epilogue stores in flight while the next tile starts), at the
    d = 768 of the workloads.  128 experts of 64..128 rows, some with a second slot; with and without the gather."""
    E, d, F = 128, 768, 1536
    rng = np.random.default_rng(11)
    rows, experts = [], []
    for e in range(E):
        rows.append(int(rng.integers(64, 129)))
        experts.append(e)
        if e % 17 == 3:
            rows.append(int(rng.integers(64, 129)))
            experts.append(e)
    so, se = _slots_for(rows, experts)
    K = int(so[-1])
    T = K + 2
    assert T >= 4096 and T >= 64 * len(rows) and len(rows) * (F // 256) > 3 * 256
    x = synth.normal_tensor((T, d), 1.0, [81], synth.BF16)
    w1 = synth.normal_tensor((E, d, F), 0.05, [82], synth.BF16)
    w2 = synth.normal_tensor((E, F, d), 0.05, [83], synth.BF16)
    ref = oracle.ffn(x, w1, w2, so, se, len(rows))
    args = (moe.moe_pack_weights(to_dev(w1)), moe.moe_pack_weights(to_dev(w2)), to_dev(so), to_dev(se),
            torch.tensor([len(rows)], dtype=torch.int32, device="cuda"), E, F)
    y = moe.moe_expert_ffn(to_dev(x), *args)
    _sync()
    assert_close(to_host(y)[:K], ref[:K], synth.BF16, "ffn bf16 short tiles, several per workgroup")
    y_off = moe.moe_expert_ffn(to_dev(x), *args, schedule=1)
    assert torch.equal(y[:K], y_off[:K])
    perm = np.random.default_rng(12).permutation(T).astype(np.int32)
    x_src = np.zeros_like(x)
    x_src[perm] = x
    y2 = moe.moe_expert_ffn(to_dev(x_src), *args, row_index=to_dev(perm))
    assert torch.equal(y[:K], y2[:K])


def test_ffn_bf16_dense_tiles_persistent():
    """More 256-row tiles than the chip has compute units, so the persistent workgroups of the tile
    kernel walk several tiles each (prefetch across tiles, epilogue stores still in flight).  The
    oracle checks sampled rows; every row must equal the experts schedule bit for bit, which runs
    the 128-column kernel alone and accumulates in the same order."""
    E, d, F = 4, 256, 512
    rows = [30000, 20000, 130, 15000, 257, 15001]
    experts = [0, 1, 1, 2, 3, 3]
    so, se = _slots_for(rows, experts)
    K = int(so[-1])
    T = K
    x = synth.normal_tensor((T, d), 1.0, [41], synth.BF16)
    w1 = synth.normal_tensor((E, d, F), 0.05, [42], synth.BF16)
    w2 = synth.normal_tensor((E, F, d), 0.05, [43], synth.BF16)
    args = (moe.moe_pack_weights(to_dev(w1)), moe.moe_pack_weights(to_dev(w2)), to_dev(so), to_dev(se),
            torch.tensor([len(rows)], dtype=torch.int32, device="cuda"), E, F)
    perm = np.random.default_rng(3).permutation(T).astype(np.int32)
    x_src = np.zeros_like(x)
    x_src[perm] = x
    y = moe.moe_expert_ffn(to_dev(x_src), *args, row_index=to_dev(perm))
    y_off = moe.moe_expert_ffn(to_dev(x), *args, schedule=1)
    _sync()
    assert torch.equal(y, y_off)
    rng = np.random.default_rng(4)
    sample = np.unique(np.concatenate([rng.choice(K, 1500, replace=False), so[:-1], so[1:] - 1,
                                       [255, 256, 29999 - 255, 29999 - 256]])).astype(np.int32)
    xs = np.zeros_like(x)
    xs[sample] = x[sample]
    ref = oracle.ffn(xs, w1, w2, so, se, len(rows), rows=sample)
    assert_close(to_host(y)[sample], ref[sample], synth.BF16, "ffn bf16 dense tiles, sampled rows")


# --------------------------------------------------------------------------- whole layer
def _run_layer_gpu(c, C, R, schedule=0, residual=0, plan_ids=None, packed=None, fuse_gather=True):
    dt = torch.bfloat16 if c["dtype"] == synth.BF16 else torch.float32
    layer = moe.MoeLayer(c["T"], c["d"], c["F"], c["E"], R, C, dt)
    x, wr, b = to_dev(c["x"]), to_dev(c["w_router"]), to_dev(c["b_router"])
    if packed is None:
        w1, w2 = to_dev(c["w1"]), to_dev(c["w2"])
        if c["dtype"] == synth.BF16:
            w1, w2 = moe.moe_pack_weights(w1), moe.moe_pack_weights(w2)
    else:
        w1, w2 = packed
    out = layer.forward(x, wr, b, w1, w2, plan_ids=plan_ids, schedule=schedule, residual=residual,
                        fuse_gather=fuse_gather)
    _sync()
    return layer, out, (w1, w2)


def _compare_layer(c, C, R, layer, out, residual=0, rows=None, plan_ids_host=None):
    """Teacher-forced comparison: ids/prob of the GPU router feed the oracle's later stages."""
    E, T = c["E"], c["T"]
    ref_rt = oracle.route(c["x"], c["w_router"], c["b_router"])
    g_idx, g_prob = to_host(layer.route_out[0]), to_host(layer.route_out[1])
    tau = (1e-5 if c["dtype"] == synth.F32 else 1e-4) * max(1.0, np.abs(ref_rt["logits"]).max())
    flips = check_ids_margin(g_idx, ref_rt["idx"], ref_rt["idx2"], ref_rt["margin"], tau, "layer route")
    same = g_idx == ref_rt["idx"]
    assert np.abs(g_prob - ref_rt["prob"])[same].max() <= 1e-4
    ref = oracle.layer(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"], C, R, residual=residual,
                       idx=g_idx, prob=g_prob, rows=rows, plan_ids=plan_ids_host)
    for k, rk in (("plan_counts", "counts"), ("replicas", "replicas"), ("slot_base", "slot_base"),
                  ("slot_expert", "slot_expert")):
        assert (to_host(layer.plan_out[k]) == ref["plan"][rk]).all(), k
    assert int(layer.plan_out["n_slots"].item()) == ref["plan"]["n_slots"]
    for k in ("counts", "kept", "expert_offset", "slot_offset", "perm", "inv"):
        assert (to_host(layer.disp_out[k]) == ref["dispatch"][k]).all(), k
    K = int(ref["dispatch"]["expert_offset"][E])
    inv = ref["dispatch"]["inv"]
    assert K + int((inv < 0).sum()) == T
    got = to_host(out)
    assert (got[inv < 0] == c["x"][inv < 0]).all()            # over-capacity tokens pass through
    if rows is None:
        assert_close(to_host(layer.y_perm)[:K], ref["y_perm"][:K], c["dtype"], "y_perm")
        assert_close(got, ref["out"], c["dtype"], "layer out")
    else:
        toks = ref["dispatch"]["perm"][rows]
        assert_close(to_host(layer.y_perm)[rows], ref["y_perm"][rows], c["dtype"], "y_perm sample")
        assert_close(got[toks], ref["out"][toks], c["dtype"], "layer out sample")
    return flips, K


@pytest.mark.parametrize("schedule", [0, 1])
@pytest.mark.parametrize("residual", [0, 1])
def test_layer_config1(schedule, residual):
    c = synth.config_inputs(1)
    layer, out, _ = _run_layer_gpu(c, c["C"], c["R"], schedule, residual, fuse_gather=bool(schedule))
    flips, K = _compare_layer(c, c["C"], c["R"], layer, out, residual)
    assert flips == 0 and K == c["T"]


@pytest.mark.parametrize("T,E,C,R", [(700, 8, 60, 3), (1500, 16, 50, 0), (2000, 128, 10, 16)])
def test_layer_bf16_small_with_drops(T, E, C, R):
    c = synth.moe_layer_inputs(T, 128, 256, E, synth.BF16, 1.1, 70 + T)
    layer, out, packed = _run_layer_gpu(c, C, R)
    fused = out.clone()
    _compare_layer(c, C, R, layer, out)
    # materialised x_perm instead of the gather fused into the first GEMM: same bits
    layer2, out2, _ = _run_layer_gpu(c, C, R, packed=packed, fuse_gather=False)
    assert torch.equal(fused, out2)
    K = int(layer2.disp_out["expert_offset"][E].item())
    perm = layer2.disp_out["perm"][:K].long()
    assert torch.equal(layer2.disp_out["x_perm"][:K], to_dev(c["x"])[perm])


def test_replication_on_and_off_give_identical_outputs_config2():
    """Same plan and capacity vector, slot schedule vs one item per logical expert."""
    c = synth.config_inputs(2)
    layer, out_on, packed = _run_layer_gpu(c, c["C"], c["R"], schedule=0)
    on = out_on.clone()
    K = int(layer.disp_out["expert_offset"][c["E"]].item())
    flips, _ = _compare_layer(c, c["C"], c["R"], layer, on)          # every kept row, every token
    print(f"config 2: {flips} near-tie flips, K={K}", flush=True)
    layer2, out_off, _ = _run_layer_gpu(c, c["C"], c["R"], schedule=1, packed=packed)
    assert torch.equal(on, out_off)
    # budget 0: the plain Switch layer keeps fewer tokens
    layer3, out_plain, _ = _run_layer_gpu(c, c["C"], 0, packed=packed)
    K0 = int(layer3.disp_out["expert_offset"][c["E"]].item())
    assert K0 < K
    _compare_layer(c, c["C"], 0, layer3, out_plain)


def test_replication_invariance_no_drops():
    """With room for every token the outputs do not depend on the replica plan."""
    c = synth.moe_layer_inputs(1500, 128, 256, 16, synth.BF16, 1.2, 123)
    layer_a, out_a, packed = _run_layer_gpu(c, 1500, 0)
    a = out_a.clone()
    hot = int(layer_a.plan_out["plan_counts"].argmax().item())
    n_hot = int(layer_a.plan_out["plan_counts"].max().item())
    assert n_hot <= 700
    # a forged prediction (two experts, 750 ids each -> a second slot for both) is wrong about the load;
    # the slot capacity is chosen so that one slot already holds the busiest expert, so nothing may
    # drop whatever the plan hands out, and the outputs must not move
    forged = to_dev((np.arange(1500) % 2).astype(np.int32))
    layer_b, out_b, _ = _run_layer_gpu(c, 700, 40, plan_ids=forged, packed=packed)
    assert to_host(layer_b.plan_out["replicas"]).tolist() == [2, 2] + [1] * 14
    assert int(layer_b.disp_out["expert_offset"][16].item()) == 1500
    assert torch.equal(a, out_b)
    all_hot = torch.full((1500,), hot, dtype=torch.int32, device="cuda")
    layer_c, out_c, _ = _run_layer_gpu(c, 700, 9, plan_ids=all_hot, packed=packed)
    assert int(layer_c.plan_out["replicas"][hot].item()) == 3      # ceil(1500/700) slots
    assert int(layer_c.disp_out["expert_offset"][16].item()) == 1500
    assert torch.equal(a, out_c)


# --------------------------------------------------------------------------- empty batch
def test_empty_batch_through_every_call():
    """T = 0: the index calls write the tables of a batch without tokens (checked against the
    oracle), the tensor calls accept NULL data pointers and enqueue nothing."""
    E, R, C, d, F = 8, 3, 5, 64, 128
    none_i = torch.empty(0, dtype=torch.int32, device="cuda")
    x = torch.empty(0, d, dtype=torch.float32, device="cuda")
    w_r = to_dev(synth.normal_tensor((d, E), 0.02, [1], synth.F32))
    idx, prob, _ = moe.moe_route(x, w_r)
    assert idx.numel() == 0 and prob.numel() == 0
    ref_pl = oracle.plan(np.zeros(0, np.int32), E, R, C)
    pl = moe.replica_plan(none_i, E, R, C)
    assert (to_host(pl["plan_counts"]) == ref_pl["counts"]).all()
    for k in ("replicas", "slot_base", "slot_expert"):
        assert (to_host(pl[k]) == ref_pl[k]).all(), k
    assert int(pl["n_slots"].item()) == ref_pl["n_slots"]
    ref_dp = oracle.dispatch(np.zeros((0, d), np.float32), np.zeros(0, np.int32), ref_pl["replicas"], E, C, E + R)
    dp = moe.moe_dispatch(x, none_i, pl["replicas"], E, C, E + R)
    for k in ("counts", "kept", "expert_offset", "slot_offset"):
        assert (to_host(dp[k]) == ref_dp[k]).all(), k
    w1 = to_dev(synth.normal_tensor((E, d, F), 0.02, [2], synth.F32))
    w2 = to_dev(synth.normal_tensor((E, F, d), 0.02, [3], synth.F32))
    y = moe.moe_expert_ffn(x, w1, w2, dp["slot_offset"], pl["slot_expert"], pl["n_slots"], E, F, max_slots=E + R)
    assert y.shape == (0, d)
    out = moe.moe_combine(y, x, none_i, prob, residual=1)
    assert out.shape == (0, d)
    _sync()
