#!/usr/bin/env python3
"""Benchmark of the replicated top-1 MoE layer forward on one MI355X.

A step = one pass of the whole layer path on one resident batch of synthetic tokens:
moe_route -> moe_plan_dispatch (replica plan + dispatch tables) -> moe_expert_ffn (rows gathered
through the permutation) -> moe_combine; the workloads with a predictor run sru_predict in front
and its ids drive the plan.  Default workload: the Switch-base-128 shaped layer (T=4096, d=768,
F=3072, E=128, capacity factor 1.25, replica budget 16, bf16 with fp32 accumulation),
Zipf(1.0)-skewed routing.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
                    [--workload cfg1|cfg2|cfg2k3|cfg3|cfg3x|cfg4|cfg4b|cfg5|cfg5stack]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch (fetched + written) of the two FFN product kernels, from two rocprofv3 --pmc
# runs of this script per workload (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter reads
# for a plain 1 GiB copy (fetch x1.9999, write x1.0000); figures and commands in profiles/ (moe_layer_*.md,
# sru*_cfg3*.md).  Counters cannot be read inside a normal run, so the values are carried here and are
# refreshed, with those files, whenever these kernels change (roofline.traffic_source says so in the line).
PMC_TRAFFIC_BYTES = {
    "cfg1": {"ffn_gemm1": 1.26e6 + 0.52e6, "ffn_gemm2": 1.31e6 + 0.13e6},
    "cfg2": {"ffn_gemm1": 630.59e6 + 15.12e6, "ffn_gemm2": 621.04e6 + 3.78e6},
    "cfg2k3": {"ffn_gemm1": 696.79e6 + 52.2e6, "ffn_gemm2": 744.75e6 + 13.05e6},
    "cfg3": {"ffn_gemm1": 639.41e6 + 24.1e6, "ffn_gemm2": 638.22e6 + 6.02e6},
    "cfg3x": {"ffn_gemm1": 637.84e6 + 23.25e6, "ffn_gemm2": 648.11e6 + 5.81e6},
    "cfg4": {"ffn_gemm1": 1252.87e6 + 40.63e6, "ffn_gemm2": 1231.49e6 + 10.16e6},
    "cfg4b": {"ffn_gemm1": 1243.81e6 + 63.36e6, "ffn_gemm2": 1266.47e6 + 15.84e6},
    # cfg5: every row goes through the 256 x 256 tile kernel; cfg5stack runs six such layers per step
    "cfg5": {"ffn_gemm1": 2073.34e6 + 402.65e6, "ffn_gemm2": 2237.45e6 + 100.66e6},
    "cfg5stack": {"ffn_gemm1": 2073.34e6 + 402.65e6, "ffn_gemm2": 2237.45e6 + 100.66e6},
}


def _to_dev(a):
    import torch
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def _workload(name):
    import synth
    if name == "cfg1":
        # the small fp32 case the oracle evaluates whole in milliseconds: cache-resident, launch-latency bound
        c = synth.config_inputs(1)
        return c, c["C"], "tiny fp32 layer T=512 d=64 F=256 E=8 C=80 R=4 Zipf(1.2) (cache-resident; latency only)"
    if name == "cfg2":
        c = synth.config_inputs(2)
        return c, c["C"], "Switch-base-128 layer T=4096 d=768 F=3072 E=128 CF=1.25 R=16 Zipf(1.0)"
    if name == "cfg3":
        # The predictor runs in front of a workload-2 shaped layer and its ids drive the replica plan.  The
        # layer's tokens and router are planted once the predictor's ids are known (main), so that the
        # router agrees with the prediction on 85 % of the tokens and draws the rest from Zipf(1.0).
        c = synth.config_inputs(3)
        return c, c["C"], ("2-layer SRU predictor (B=8 L=512 768->256, head 128) + Switch-base-128 layer "
                           "T=4096 d=768 F=3072 E=128 CF=1.25 R=16, router agrees with the prediction on 85% of tokens")
    if name == "cfg3x":
        # the paper's predictor size: 10 SRU layers and the sparsemax attention in front of the head
        c = synth.config_inputs(3)
        c["sru"] = synth.sru_inputs(8, 512, 768, 256, 10, 128, synth.BF16, synth.workloads.SEED0 + 33, w_std=0.05)
        c["sru"]["attention"] = True
        return c, c["C"], ("10-layer SRU predictor with sparsemax attention (B=8 L=512 768->256, head 128) + "
                           "Switch-base-128 layer T=4096 d=768 F=3072 E=128 CF=1.25 R=16, router agrees with the "
                           "prediction on 85% of tokens")
    if name == "cfg2k3":
        # top-3 routing on the workload-2 layer: 3 x 4096 assignments, slot capacity scaled by k
        c = synth.config_inputs(2)
        c["top_k"] = 3
        return c, 3 * c["C"], "Switch-base-128 layer, top-3 routing: T=4096 d=768 F=3072 E=128 CF=1.25 R=16 Zipf(1.0)"
    if name == "cfg4":
        c = synth.config_inputs(4)
        return c, c["C"], "Switch-base-256 layer T=16384 d=768 F=3072 E=256 CF=1.0 R=32 Zipf(1.1)"
    if name == "cfg4b":
        c = synth.config_inputs(4)
        return c, c["C_alt"], "Switch-base-256 layer T=16384 d=768 F=3072 E=256 CF=2.0 R=32 Zipf(1.1)"
    if name == "cfg5":
        c = synth.config_inputs(5)
        c.update(c["layers"][0])
        c["residual"] = 1
        return c, c["C"], ("extreme skew, one layer of the stack (with its residual connection): T=65536 E=256 "
                           "CF=4.0 R=64, 50% hot expert")
    if name == "cfg5stack":
        c = synth.config_inputs(5)
        c["residual"] = 1
        c["stack"] = True
        return c, c["C"], (f"extreme skew, the whole stack: {len(c['layers'])} MoE layers per step with independent "
                           "weights and a residual connection between them, T=65536 E=256 CF=4.0 R=64, 50% hot expert")
    raise SystemExit(f"unknown workload {name}")


def _time_steps(step, steps):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def _cpu_baseline(c, C, R, budget_s=20.0, serial_leg=True):
    """The oracle as it stands, on the host cores: router, plan, dispatch and combine on the
    whole batch, the expert FFN on a sample of kept rows sized to ~budget_s, scaled to K."""
    import oracle
    T, E = c["T"], c["E"]
    k = c.get("top_k", 1)
    oracle.route(c["x"][:64], c["w_router"], c["b_router"])      # untimed: loads the library, starts its threads
    t0 = time.perf_counter()
    if k == 1:
        rt = oracle.route(c["x"], c["w_router"], c["b_router"])
        pl = oracle.plan(rt["idx"], E, R, C)
        dp = oracle.dispatch(c["x"], rt["idx"], pl["replicas"], E, C, E + R)
    else:
        from oracle import topk
        rt = oracle.route_topk(c["x"], c["w_router"], c["b_router"], k)
        ids = rt["idx"].reshape(-1)
        pl = oracle.plan(ids, E, R, C)
        dp = oracle.dispatch(topk.assignment_rows(c["x"], k), ids, pl["replicas"], E, C, E + R)
    t_front = time.perf_counter() - t0
    K = int(dp["expert_offset"][E])
    rng = np.random.default_rng(0)
    probe = np.sort(rng.choice(K, size=min(K, 32), replace=False)).astype(np.int32)
    t0 = time.perf_counter()
    oracle.ffn(dp["x_perm"], c["w1"], c["w2"], dp["slot_offset"], pl["slot_expert"], pl["n_slots"], rows=probe)
    per_row = (time.perf_counter() - t0) / len(probe)
    n = int(max(32, min(K, budget_s / max(per_row, 1e-9))))
    rows = np.sort(rng.choice(K, size=n, replace=False)).astype(np.int32)
    t0 = time.perf_counter()
    y = oracle.ffn(dp["x_perm"], c["w1"], c["w2"], dp["slot_offset"], pl["slot_expert"], pl["n_slots"], rows=rows)
    t_ffn = (time.perf_counter() - t0) * (K / n)
    t0 = time.perf_counter()
    if k == 1:
        oracle.combine(y, c["x"], dp["inv"], rt["prob"], int(c.get("residual", 0)))
    else:
        oracle.combine_topk(y, c["x"], dp["inv"].reshape(k, T), rt["weight"], int(c.get("residual", 0)))
    t_back = time.perf_counter() - t0
    total = t_front + t_ffn + t_back
    res = dict(value=T / total, unit="tokens/s", cores=oracle.num_threads(), kind="oracle",
               sample=f"router, plan, dispatch, combine on all {T} tokens; expert FFN on {n} of the {K} kept "
                      f"rows, its time scaled by {K}/{n}")
    if serial_leg and total * res["cores"] < 30.0:
        # the same work once more on one thread (small workloads only, where that stays within seconds)
        cores = oracle.num_threads()
        oracle.set_num_threads(1)
        try:
            one = _cpu_baseline(c, C, R, budget_s, serial_leg=False)
        finally:
            oracle.set_num_threads(cores)
        res["value_1_thread"] = round(one["value"], 1)
    return res


def _ffn_split(moe, x, w1, w2, T, d, F, E, R, C, counts):
    """moe_expert_ffn alone on slot tables made from this batch's expert loads: the busiest expert's rows only
    (cut into slots of C rows), all other experts only, both, and as many rows spread evenly over all experts.
    Event-timed per product.  Input construction only; every product runs in the library."""
    import torch
    hot = int(np.argmax(counts))

    def slots_of(expert_rows):
        rows, experts = [], []
        for e, n in expert_rows:
            n = int(min(n, T))
            r = max(1, -(-n // C))
            q, rem = divmod(n, r)
            for k in range(r):
                rows.append(q + (k < rem))
                experts.append(e)
        return rows, experts

    cases = {
        "hot_expert_only": slots_of([(hot, counts[hot])]),
        "other_experts_only": slots_of([(e, counts[e]) for e in range(E) if e != hot]),
        "both": slots_of([(e, counts[e]) for e in range(E)]),
        "uniform_256_rows_per_expert": ([min(256, T // E)] * E, list(range(E))),
        "uniform_64_rows_per_expert": ([min(64, T // E)] * E, list(range(E))),
    }
    out = {}
    for name, (rows, experts) in cases.items():
        P = len(rows)
        max_slots = max(P, E + R)
        so = np.zeros(max_slots + 1, np.int32)
        so[1:P + 1] = np.cumsum(rows)
        so[P + 1:] = so[P]
        se = np.full(max_slots, -1, np.int32)
        se[:P] = experts
        so_t, se_t = torch.from_numpy(so).cuda(), torch.from_numpy(se).cuda()
        ns = torch.tensor([P], dtype=torch.int32, device="cuda")
        y = torch.empty_like(x)
        ws = torch.empty(moe.lib().moe_expert_ffn_workspace_bytes(T, max_slots, d, F, moe.MOE_BF16), dtype=torch.uint8,
                         device="cuda")
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(10)]
        for t in evs:
            for e in t:
                e.record()
        for i in range(10):
            moe.moe_expert_ffn(x, w1, w2, so_t, se_t, ns, E, F, max_slots=max_slots, out=y, ws=ws, events=evs[i])
        torch.cuda.synchronize()
        g1 = float(np.mean([t[0].elapsed_time(t[1]) for t in evs[2:]]))
        g2 = float(np.mean([t[1].elapsed_time(t[2]) for t in evs[2:]]))
        K = int(so[P])
        active = len(set(experts))
        out[name] = {"rows": K, "slots": P, "experts": active, "ffn_gemm1_ms": round(g1, 5), "ffn_gemm2_ms": round(g2, 5),
                     "gemm1_tflops": round(2.0 * K * d * F / g1 / 1e9, 1),
                     "gemm1_algorithmic_GBs": round((active * d * F * 2 + K * d * 2 + K * F * 2) / g1 / 1e6, 1)}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay timing")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured ceilings (a 1 GiB read stream, plain and non-temporal, and a "
                         "matrix-instruction loop with the dense tile's instruction mix)")
    ap.add_argument("--pmc-calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a reference dispatch of known size for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--materialize-gather", action="store_true",
                    help="top-1 workloads: moe_dispatch copies the kept rows into x_perm (dispatch_gather_kernel) and "
                         "the first product reads that copy, instead of gathering through the permutation")
    ap.add_argument("--ffn-split", action="store_true",
                    help="also time moe_expert_ffn alone on synthetic slot tables cut from this workload's shape: the "
                         "hot expert's slots only, the other experts only, both, and uniform slots (where the two "
                         "products' time goes when matrix-bound and weight-streaming tiles share a launch)")
    ap.add_argument("--modes", default="on,off_same_plan,off_budget0",
                    help="replication modes to time besides 'on' (comma list)")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        raise SystemExit(2)

    import torch
    import paper_2605_11537_amd as moe
    moe.lib()
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")

    c, C, desc = _workload(a.workload)
    T, d, F, E, R = c["T"], c["d"], c["F"], c["E"], c["R"]
    sru = None
    if "sru" in c:
        import synth
        s_ = c["sru"]
        sru_w = moe.SruWeights([_to_dev(w) for w in s_["w_cat"]], None, None, _to_dev(s_["w_head"]), None, pack=True,
                               attention=bool(s_.get("attention", False)))
        emb = _to_dev(s_["emb"])
        pred = torch.empty(T, dtype=torch.int32, device="cuda")
        sru_ws = torch.empty(moe.lib().sru_predict_workspace_bytes(__import__("ctypes").byref(sru_w.c), s_["B"],
                                                                   s_["L"], moe.MOE_BF16), dtype=torch.uint8,
                             device="cuda")
        sru = (emb, sru_w, pred, sru_ws)
        if "x" not in c:
            # the layer of this workload: ids that agree with the predictor's on `agree` of the tokens, planted
            # as the largest router logit of their token (pure input generation; no method arithmetic)
            moe.sru_predict(emb, sru_w, out=pred, ws=sru_ws)
            torch.cuda.synchronize()
            seed = synth.workloads.SEED0 + 3
            z = synth.mix_ids(pred.cpu().numpy(), E, c["agree"], c["zipf_s"], seed)
            lay = synth.planted_layer_inputs(z, d, F, E, c["dtype"], seed, c["alpha"], c["beta"], 1)
            c.update({k: v for k, v in lay.items() if k != "layers"})
            c.update(lay["layers"][0])
    fp32 = c["x"].dtype == np.float32
    dt = torch.float32 if fp32 else torch.bfloat16
    x = _to_dev(c["x"])
    RL = moe.LAYOUT_PLAIN if fp32 else moe.LAYOUT_PACKED
    layer_inputs = c["layers"] if c.get("stack") else [c]
    W = []                                   # per layer: router matrix, router bias, W1, W2 on the device
    for lw in layer_inputs:
        if fp32:
            W.append((_to_dev(lw["w_router"]), _to_dev(lw["b_router"]), _to_dev(lw["w1"]), _to_dev(lw["w2"])))
        else:
            # static weights are packed once, outside the timed region (router included)
            W.append((moe.moe_pack_weights(_to_dev(lw["w_router"])[None].contiguous())[0], _to_dev(lw["b_router"]),
                      moe.moe_pack_weights(_to_dev(lw["w1"])), moe.moe_pack_weights(_to_dev(lw["w2"]))))
        torch.cuda.synchronize()
    n_layers = len(W)
    wr, b, w1, w2 = W[0]
    # a stack hands the output of one layer to the next: two buffers in turn
    outs = [torch.empty(T, d, dtype=dt, device="cuda") for _ in range(2)] if n_layers > 1 else None

    if a.materialize_gather and c.get("top_k", 1) != 1:
        raise SystemExit("--materialize-gather is for the top-1 workloads")

    def chain(lay, schedule, marks=None, **kw):
        if a.materialize_gather:
            kw["fuse_gather"] = False
        cur = x
        for l, (wr_l, b_l, w1_l, w2_l) in enumerate(W):
            ffn_events = kw.pop("ffn_events", None) if l == 0 else None     # first layer of a stack only
            cur = lay.forward(cur, wr_l, b_l, w1_l, w2_l, schedule=schedule, router_layout=RL, residual=RES,
                              out=None if outs is None else outs[l % 2], marks=marks if l == 0 else None,
                              ffn_events=ffn_events, **kw)
        return cur

    top_k = c.get("top_k", 1)
    RES = int(c.get("residual", 0))      # the layers of the workload-5 stack add their input (residual connection)
    if top_k == 1:
        layer = moe.MoeLayer(T, d, F, E, R, C, dt)
        layer0 = moe.MoeLayer(T, d, F, E, 0, C, dt)          # budget 0: the plain Switch layer
    else:
        layer = moe.MoeLayerTopK(T, d, F, E, top_k, R, C, dt)
        layer0 = moe.MoeLayerTopK(T, d, F, E, top_k, 0, C, dt)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(a.steps)]
    for trio in evs:
        for e in trio:
            e.record()                                   # creates the underlying hipEvent
    it = {"i": 0, "timed": False}

    def step_on():
        plan_ids = None
        if sru is not None:
            plan_ids, _ = moe.sru_predict(sru[0], sru[1], out=sru[2], ws=sru[3])
        kw = {} if plan_ids is None else {"plan_ids": plan_ids}
        if it["timed"]:
            kw["ffn_events"] = evs[it["i"]]
            it["i"] += 1
        chain(layer, moe.SCHEDULE_SLOTS, **kw)

    def _plan_kw():
        # with a predictor in front, every mode runs it and plans from its ids
        if sru is None:
            return {}
        return {"plan_ids": moe.sru_predict(sru[0], sru[1], out=sru[2], ws=sru[3])[0]}

    def step_off_same_plan():
        chain(layer, moe.SCHEDULE_EXPERTS, **_plan_kw())

    def step_off_budget0():
        chain(layer0, moe.SCHEDULE_SLOTS, **_plan_kw())

    for _ in range(a.warmup):
        step_on()
    ms_on = _time_steps(step_on, a.steps)           # headline: K clean steps
    # second pass over the same K steps, the two FFN GEMM kernels bracketed by HIP events on the
    # launch stream (recording an event between kernels costs a few us, so it is kept out of the
    # headline pass)
    it["timed"] = True
    ms_on_events = _time_steps(step_on, a.steps)
    it["timed"] = False
    g1 = float(np.mean([t[0].elapsed_time(t[1]) for t in evs]))
    g2 = float(np.mean([t[1].elapsed_time(t[2]) for t in evs]))

    # third pass: events between the calls of every step -> per-call times, and the spread over steps
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(a.steps)]

    def step_marked(i):
        m = marks[i]
        m[5].record()                                  # step start (before the predictor, if any)
        plan_ids = None
        if sru is not None:
            plan_ids, _ = moe.sru_predict(sru[0], sru[1], out=sru[2], ws=sru[3])
        kw = {} if plan_ids is None else {"plan_ids": plan_ids}
        chain(layer, moe.SCHEDULE_SLOTS, marks=m[:5], **kw)       # the marks sit in the first layer of a stack

    end_ev = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    for i in range(a.steps):
        step_marked(i)
    end_ev.record()
    torch.cuda.synchronize()
    call_names = ("sru_predict", "moe_route", "moe_plan_dispatch", "moe_expert_ffn", "moe_combine")
    spans = ((5, 0), (0, 1), (1, 2), (2, 3), (3, 4))
    per_call = {n: round(float(np.median([m[i].elapsed_time(m[j]) for m in marks])), 5)
                for n, (i, j) in zip(call_names, spans) if n != "sru_predict" or sru is not None}
    step_ms = [marks[i][5].elapsed_time(marks[i + 1][5]) for i in range(a.steps - 1)]
    step_ms.append(marks[-1][5].elapsed_time(end_ev))

    kept = layer.disp_out["kept"].cpu().numpy()
    counts = layer.disp_out["counts"].cpu().numpy().astype(np.int64)
    replicas = layer.plan_out["replicas"].cpu().numpy()
    # the realised skew of this batch (a description of the input, taken from the library's own tables)
    routing = {"assignments": int(counts.sum()), "max_expert_share": round(float(counts.max() / max(1, counts.sum())), 4),
               "experts_over_slot_capacity": int((counts > C).sum()),
               "replicas_wanted": int(np.maximum(0, -(-counts // C) - 1).sum()),
               "replicas_granted": int(replicas.sum() - E)}
    if sru is not None:
        routing["router_agrees_with_prediction"] = round(float((layer.route_out[0] == sru[2]).float().mean().item()), 4)
    K = int(kept.sum())
    active = int((kept > 0).sum())
    n_slots = int(layer.plan_out["n_slots"].item())
    esz = 4 if fp32 else 2
    bytes_g1 = active * d * F * esz + K * d * esz + K * F * esz
    bytes_g2 = active * F * d * esz + K * F * esz + K * d * esz
    flops = 2.0 * K * d * F
    dom = ("ffn_gemm1", g1, bytes_g1) if g1 >= g2 else ("ffn_gemm2", g2, bytes_g2)
    ach = dom[2] / (dom[1] * 1e-3) / 1e9                         # GB/s of algorithmic bytes
    tfl = flops / (dom[1] * 1e-3) / 1e12                         # TFLOP/s of the same launch
    # Which roof binds the dominant launch: the time its algorithmic bytes take at the HBM peak against the
    # time its flops take at the matrix-core peak (fp32 workload 1: the vector fp32 peak stands in)
    peak_tfl = MFMA_BF16_PEAK_TFLOPS if not fp32 else 157.3
    t_hbm, t_mma = dom[2] / (HBM_PEAK_GBS * 1e9), flops / (peak_tfl * 1e12)
    bound = "hbm" if t_hbm >= t_mma else ("mfma" if not fp32 else "alu")
    traffic = PMC_TRAFFIC_BYTES.get(a.workload, {}).get(dom[0])
    if bound == "hbm":
        roofline = dict(bound="hbm", kernel=dom[0], achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=round(ach / HBM_PEAK_GBS, 4))
    else:
        roofline = dict(bound=bound, kernel=dom[0], achieved=round(tfl, 1), peak=peak_tfl, unit="TFLOP/s",
                        frac=round(tfl / peak_tfl, 4))
    roofline.update(traffic=traffic,
                    traffic_source=None if traffic is None else f"profiles/ (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE of {dom[0]}, "
                                                              "scaled by a 1 GiB copy; a constant refreshed with the kernels)",
                    avg_ms=round(dom[1], 5), algorithmic_bytes=int(dom[2]), flops=int(flops),
                    ideal_ms_at_hbm_peak=round(t_hbm * 1e3, 5), ideal_ms_at_matrix_peak=round(t_mma * 1e3, 5),
                    hbm_frac_of_peak=round(ach / HBM_PEAK_GBS, 4),
                    ffn_gemm1_ms=round(g1, 5), ffn_gemm2_ms=round(g2, 5),
                    ffn_mfma_tflops=round(2 * flops / ((g1 + g2) * 1e-3) / 1e12, 2),
                    ffn_mfma_frac_of_bf16_peak=round(2 * flops / ((g1 + g2) * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4))
    if not a.no_ceilings:
        # what this machine delivers to a kernel of the same shape: a pure read stream, a pure matrix-instruction loop
        cl = moe.measure_ceilings()
        roofline["measured_peak"] = cl
        if bound == "hbm":
            roofline["frac_of_measured_peak"] = round(ach / cl["hbm_read_nontemporal_GBs"], 4)
        elif bound == "mfma":
            roofline["frac_of_measured_peak"] = round(tfl / cl["mfma_bf16_operands_from_lds_TFLOPs"], 4)

    # the same step captured once into a HIP graph and replayed (the library allocates nothing, records no
    # memset and never synchronises, so the whole chain of launches is capturable)
    graph_ms = None
    if not a.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step_on()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step_on()
        for _ in range(a.warmup):
            g.replay()
        graph_ms = _time_steps(g.replay, a.steps)

    pipeline = None
    if sru is not None:
        # the paper's two threads as two streams: predictor + plan of batch i+1 under the layer of batch i
        pipe = moe.MoePipeline(layer, sru[1], c["sru"]["B"], c["sru"]["L"])
        pipe.predict(sru[0])

        def step_pipelined():
            pipe.predict(sru[0])
            pipe.forward(x, wr, b, w1, w2, schedule=moe.SCHEDULE_SLOTS, router_layout=RL, residual=RES)

        for _ in range(a.warmup):
            step_pipelined()
        ms_pipe = _time_steps(step_pipelined, a.steps)
        pipeline = {"ms_per_step": round(ms_pipe, 5), "tokens_per_s": round(T / (ms_pipe * 1e-3), 1),
                    "note": "sru_predict + replica_plan of the next batch on a second stream"}

    modes = {"on": round(T / (ms_on * 1e-3), 1)}
    extra_ms = {"on": round(ms_on, 5)}
    for name, fn in (("off_same_plan", step_off_same_plan), ("off_budget0", step_off_budget0)):
        if name in a.modes.split(","):
            for _ in range(max(2, a.warmup // 2)):
                fn()
            ms = _time_steps(fn, max(10, a.steps // 2))
            modes[name] = round(T / (ms * 1e-3), 1)
            extra_ms[name] = round(ms, 5)
    kept0 = int(layer0.disp_out["kept"].sum().item()) if "off_budget0" in modes else None
    # tokens that actually went through an expert, per second: "on" and "off_same_plan" keep the same K rows,
    # budget 0 keeps fewer (less work per input token)
    kept_rate = {m: round((kept0 if m == "off_budget0" else K) / (extra_ms[m] * 1e-3), 1) for m in modes}

    if a.pmc_calibration_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ffn_split = None
    if a.ffn_split and not fp32 and top_k == 1:
        ffn_split = _ffn_split(moe, x, w1, w2, T, d, F, E, R, C, counts)

    cpu = None
    if not a.no_cpu_baseline and sru is None:
        cpu = _cpu_baseline(c, C, R)
        cpu["value"] = round(cpu["value"], 1)
    # (with a predictor in front, the layer's inputs were planted from the library's own predictions, and the
    # oracle is never fed anything that came out of the HIP path: its baseline is the one of workload cfg2)

    line = {
        # the matrix-core share of peak that the metric's name asks for is roofline.ffn_mfma_frac_of_bf16_peak
        "metric": f"MoE-layer tokens/sec (route+dispatch+FFN+combine), MFMA %peak, E={E} d={d}",
        "value": modes["on"], "unit": "tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_on, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32" if fp32 else "bf16", "data": "synthetic",
        "config": {"workload": desc, "name": a.workload, "T": T, "d_model": d, "d_ff": F, "experts": E,
                   "top_k": top_k, "slot_capacity": C, "replica_budget": R, "kept_tokens": K, "active_experts": active,
                   "slots": n_slots, "replication": "on (slot schedule)", "residual": RES, "layers_per_step": n_layers,
                   "gather": "materialized by moe_dispatch" if a.materialize_gather else "fused into the first product",
                   "routing": routing},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "replication_modes_tokens_per_s": modes,
        "replication_modes_ms": extra_ms,
        "kept_tokens_per_s": kept_rate,
        "ms_per_step_with_kernel_events": round(ms_on_events, 5),
        # from the pass with events between the calls (they cost a few us per step)
        "ms_per_step_median_with_call_events": round(float(np.median(step_ms)), 5), "ms_per_step_min_with_call_events": round(float(np.min(step_ms)), 5),
        "per_call_ms_median": per_call,
        "ms_per_step_hip_graph_replay": None if graph_ms is None else round(graph_ms, 5),
        "kept_tokens_budget0": kept0,
    }
    if pipeline is not None:
        line["two_stream_pipeline"] = pipeline
    if ffn_split is not None:
        line["ffn_split"] = ffn_split
    print(json.dumps(line))


if __name__ == "__main__":
    main()
