"""GPU parity of sru_predict against the CPU oracle, and the predictor-driven layer."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import assert_close, check_ids_margin, to_dev, to_host

pytestmark = pytest.mark.gpu


def _weights(moe, s):
    return moe.SruWeights([to_dev(w) for w in s["w_cat"]], [to_dev(b) for b in s["b_f"]],
                          [to_dev(b) for b in s["b_r"]], to_dev(s["w_head"]), to_dev(s["b_head"]))


# Fixed in advance, independent of what a run measures: the logits may be off by at most
# LOGIT_TOL * max|logit| (activations are rounded to bf16 between layers; the matrix cores sum in binary32 in
# another order), the argmax must equal the oracle's wherever its top-2 gap exceeds TAU * max|logit| and be the
# runner-up otherwise, and at most MAX_FLIPS of the predictions may be such near-ties.
LOGIT_TOL = 5e-3
TAU = 5e-3
MAX_FLIPS = 0.005


def _check_prediction(got, lg, ref, what):
    scale = np.abs(ref["logits"]).max()
    err = np.abs(lg - ref["logits"]).max()
    assert err <= LOGIT_TOL * scale, f"{what}: logits off by {err / scale:.3e} of the scale"
    flips = check_ids_margin(got, ref["pred"], ref["idx2"], ref["margin"], TAU * scale, what)
    assert flips <= max(1, int(MAX_FLIPS * got.size)), f"{what}: {flips} of {got.size} predictions differ"
    return err, scale, flips


def _compare(moe, s, what):
    ref = oracle.sru(s["emb"], s["w_cat"], s["b_f"], s["b_r"], s["w_head"], s["b_head"])
    pred, logits = moe.sru_predict(to_dev(s["emb"]), _weights(moe, s), want_logits=True)
    torch.cuda.synchronize()
    lg = to_host(logits).astype(np.float64)
    got = to_host(pred)
    err, scale, flips = _check_prediction(got, lg, ref, what)
    diff = got != ref["pred"]
    print(f"{what}: max logit err {err:.2e} (scale {scale:.2f}), {int(diff.sum())} near-tie flips", flush=True)
    if s["n_out"] in (128, 256):
        # weights packed once by the caller: same kernels, same bits
        wp = moe.SruWeights([to_dev(w) for w in s["w_cat"]], [to_dev(b) for b in s["b_f"]],
                            [to_dev(b) for b in s["b_r"]], to_dev(s["w_head"]), to_dev(s["b_head"]), pack=True)
        pred2, logits2 = moe.sru_predict(to_dev(s["emb"]), wp, want_logits=True)
        assert torch.equal(pred, pred2) and torch.equal(logits, logits2)
    return got, ref


@pytest.mark.parametrize("B,L,n_in,n_h,layers,n_out,bias", [
    (3, 70, 192, 128, 2, 24, 0.3),     # ragged chunks, 4-block first layer, generic head
    (2, 16, 128, 128, 3, 128, 0.0),    # equal widths (highway = x), MFMA head
    (5, 513, 192, 128, 1, 256, 0.2),   # L not a multiple of the chunk count
    (1, 1, 128, 128, 1, 8, 0.1),
    (4, 128, 256, 128, 10, 128, 0.1),  # the depth the paper uses (10 layers)
    (2, 1500, 128, 128, 2, 8, 0.1),    # chunks longer than the register-resident scan holds
    (8, 96, 128, 256, 2, 8, 0.1),      # a multiple of 8 sequences: whole sequences per XCD in the layer kernel
    (16, 40, 64, 128, 1, 24, 0.0),
])
def test_sru_small(B, L, n_in, n_h, layers, n_out, bias):
    import paper_2605_11537_amd as moe
    s = synth.sru_inputs(B, L, n_in, n_h, layers, n_out, synth.BF16, 500 + L, bias_std=bias, w_std=0.08)
    _compare(moe, s, f"sru B={B} L={L}")


@pytest.mark.parametrize("B,L,n_in,n_h,layers,n_out", [
    (3, 70, 192, 128, 2, 24),        # ragged: L not a multiple of the 32-row tile nor of the 64-lane chunks
    (2, 512, 128, 256, 2, 128),      # the benchmark's sequence length and width
    (1, 1024, 128, 128, 1, 8),       # longest sequence the score tile holds
    (5, 1, 128, 128, 1, 8),          # one position per sequence: it attends to itself, z = 2h
    (8, 100, 128, 256, 1, 8),        # a multiple of 8 sequences: whole sequences per XCD in the attention kernel
])
def test_sru_with_sparsemax_attention(B, L, n_in, n_h, layers, n_out):
    """The attention variant of the predictor against the oracle: logits and predictions under the same
    fixed bounds and near-tie rule as without it."""
    import paper_2605_11537_amd as moe
    s = synth.sru_inputs(B, L, n_in, n_h, layers, n_out, synth.BF16, 700 + L, bias_std=0.2, w_std=0.08)
    ref = oracle.sru_attention(s["emb"], s["w_cat"], s["b_f"], s["b_r"], s["w_head"], s["b_head"])
    w = moe.SruWeights([to_dev(a) for a in s["w_cat"]], [to_dev(a) for a in s["b_f"]], [to_dev(a) for a in s["b_r"]],
                       to_dev(s["w_head"]), to_dev(s["b_head"]), attention=True)
    pred, logits = moe.sru_predict(to_dev(s["emb"]), w, want_logits=True)
    torch.cuda.synchronize()
    lg = to_host(logits).astype(np.float64)
    got = to_host(pred)
    err, scale, flips = _check_prediction(got, lg, ref, f"attention B={B} L={L}")
    diff = got != ref["pred"]
    # without the attention the same weights give different logits (the option is really on)
    w0 = moe.SruWeights([to_dev(a) for a in s["w_cat"]], [to_dev(a) for a in s["b_f"]], [to_dev(a) for a in s["b_r"]],
                        to_dev(s["w_head"]), to_dev(s["b_head"]))
    _, logits0 = moe.sru_predict(to_dev(s["emb"]), w0, want_logits=True)
    assert not torch.equal(logits, logits0)
    print(f"attention B={B} L={L}: max logit err {err:.2e} (scale {scale:.2f}), {int(diff.sum())} near-tie flips", flush=True)


def test_sru_config3_and_predictor_driven_layer():
    import paper_2605_11537_amd as moe
    c0 = synth.config_inputs(3)
    got, ref = _compare(moe, c0["sru"], "sru config 3")
    # the layer input is built from the ORACLE's predictions (inputs never come from the GPU)
    c = synth.config_inputs(3, pred=ref["pred"])
    E, C, R, T = c["E"], c["C"], c["R"], c["T"]
    layer = moe.MoeLayer(T, c["d"], c["F"], E, R, C, torch.bfloat16)
    x, wr, b = to_dev(c["x"]), to_dev(c["w_router"]), to_dev(c["b_router"])
    w1, w2 = moe.moe_pack_weights(to_dev(c["w1"])), moe.moe_pack_weights(to_dev(c["w2"]))
    pred_gpu = to_dev(got)
    out = layer.forward(x, wr, b, w1, w2, plan_ids=pred_gpu)
    torch.cuda.synchronize()
    g_idx, g_prob = to_host(layer.route_out[0]), to_host(layer.route_out[1])
    rt = oracle.route(c["x"], c["w_router"], c["b_router"])
    assert (g_idx == rt["idx"]).mean() > 0.9999
    agree = (rt["idx"] == ref["pred"]).mean()
    assert 0.82 <= agree <= 0.90, agree                      # ~85% agreement by construction
    K = int(layer.disp_out["expert_offset"][E].item())
    # every kept row and every token, the oracle planning from the same predicted ids
    full = oracle.layer(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"], C, R, idx=g_idx, prob=g_prob,
                        plan_ids=got)
    assert (to_host(layer.plan_out["replicas"]) == full["plan"]["replicas"]).all()
    for k in ("counts", "kept", "expert_offset", "slot_offset", "perm", "inv"):
        assert (to_host(layer.disp_out[k]) == full["dispatch"][k]).all(), k
    assert K == int(full["dispatch"]["expert_offset"][E])
    assert_close(to_host(layer.y_perm)[:K], full["y_perm"][:K], synth.BF16, "config 3 y_perm")
    assert_close(to_host(out), full["out"], synth.BF16, "config 3 out")
    dropped = full["dispatch"]["inv"] < 0
    assert (to_host(out)[dropped] == c["x"][dropped]).all()
    print(f"config 3: router/predictor agreement {agree:.3f}, kept {K}/{T}", flush=True)


def test_two_stream_pipeline_equals_sequential():
    """Predictor + plan of batch i+1 on a second stream under the layer of batch i: every batch must
    come out bit for bit as when the same calls run one after the other on one stream.  Batches
    differ (fresh embeddings at different scales, tokens rolled) so that a plan table read too early
    or too late would show."""
    import paper_2605_11537_amd as moe
    s = synth.sru_inputs(4, 256, 128, 128, 2, 16, synth.BF16, 901, bias_std=0.2, w_std=0.08)
    T, E, d, F, C, R = 4 * 256, 16, 128, 256, 48, 6
    c = synth.moe_layer_inputs(T, d, F, E, synth.BF16, 1.1, 902)
    w = moe.SruWeights([to_dev(a) for a in s["w_cat"]], [to_dev(a) for a in s["b_f"]], [to_dev(a) for a in s["b_r"]],
                       to_dev(s["w_head"]), to_dev(s["b_head"]))
    wr, b = to_dev(c["w_router"]), to_dev(c["b_router"])
    w1, w2 = moe.moe_pack_weights(to_dev(c["w1"])), moe.moe_pack_weights(to_dev(c["w2"]))
    emb0, x0 = to_dev(s["emb"]), to_dev(c["x"])
    n_batches = 7
    embs = [emb0] + [to_dev(synth.normal_tensor((4, 256, 128), 2.0 ** (i % 3 - 1), [903, i], synth.BF16))
                     for i in range(1, n_batches)]
    xs = [torch.roll(x0, shifts=31 * i, dims=0).contiguous() for i in range(n_batches)]
    layer = moe.MoeLayer(T, d, F, E, R, C, torch.bfloat16)
    seq = []
    for i in range(n_batches):
        ids, _ = moe.sru_predict(embs[i], w)
        seq.append(layer.forward(xs[i], wr, b, w1, w2, plan_ids=ids).clone())
    torch.cuda.synchronize()
    plans = {tuple(to_host(moe.replica_plan(moe.sru_predict(e, w)[0], E, R, C)["replicas"])) for e in embs}
    assert len(plans) > 1                                   # the batches really ask for different plans
    pipe = moe.MoePipeline(layer, w, 4, 256)
    outs = []
    pipe.predict(embs[0])
    for i in range(n_batches):
        if i + 1 < n_batches:
            pipe.predict(embs[i + 1])
        outs.append(pipe.forward(xs[i], wr, b, w1, w2).clone())
    torch.cuda.synchronize()
    for i in range(n_batches):
        assert torch.equal(outs[i], seq[i]), f"batch {i}"
    # against the definition, not only against the one-stream order: the oracle runs predictor, plan and layer
    # of the first batch, of one in the middle and of the last (the router's ids and probabilities taken from
    # a one-stream run of the library, the predictor's ids under the fixed near-tie rule)
    for i in (0, 3, n_batches - 1):
        emb_h, x_h = to_host(embs[i]), to_host(xs[i])
        ref_p = oracle.sru(emb_h, s["w_cat"], s["b_f"], s["b_r"], s["w_head"], s["b_head"])
        ids_g, lg_g = moe.sru_predict(embs[i], w, want_logits=True)
        _check_prediction(to_host(ids_g), to_host(lg_g).astype(np.float64), ref_p, f"pipeline batch {i}")
        r_idx, r_prob, _ = moe.moe_route(xs[i], wr, b)
        rt = oracle.route(x_h, c["w_router"], c["b_router"])
        check_ids_margin(to_host(r_idx), rt["idx"], rt["idx2"], rt["margin"],
                         1e-4 * max(1.0, np.abs(rt["logits"]).max()), f"pipeline batch {i} route")
        ref = oracle.layer(x_h, c["w_router"], c["b_router"], c["w1"], c["w2"], C, R, idx=to_host(r_idx),
                           prob=to_host(r_prob), plan_ids=to_host(ids_g))
        assert_close(to_host(outs[i]), ref["out"], synth.BF16, f"pipeline batch {i} out")
        dropped = ref["dispatch"]["inv"] < 0
        assert dropped.any() and (to_host(outs[i])[dropped] == x_h[dropped]).all()
    with pytest.raises(RuntimeError):
        pipe.forward(xs[0], wr, b, w1, w2)                  # nothing predicted is waiting
