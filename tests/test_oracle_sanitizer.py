"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

``oracle/sanitize_driver.c`` and ``oracle/moe_oracle.c`` are compiled into one executable with
``-fsanitize=address,undefined``; it runs the layer chain and the predictor on cases written here
(exact-size heap tensors, so one element past any of them is reported) and its outputs must equal
the ordinary build's bit for bit.  A sanitizer report makes the run fail (no recovery)."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path_factory.mktemp("san") / "oracle_sanitized")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-static-libasan", os.path.join(ROOT, "oracle", "moe_oracle.c"),
                           os.path.join(ROOT, "oracle", "sanitize_driver.c"), "-lm", "-o", exe])
    return exe


def _run(driver, tmp_path, c, s, C_, R, policy, residual):
    st = 0 if c["x"].dtype == np.float32 else 1
    T, d, F, E = c["T"], c["d"], c["F"], c["E"]
    n_layers = len(s["w_cat"]) if s else 0
    hd = np.array([T, d, F, E, C_, R, st, policy, residual, s["B"] if s else 0, s["L"] if s else 0, n_layers,
                   s["n_in"] if s else 0, s["n_hidden"] if s else 0, s["n_out"] if s else 0, 0], np.int32)
    parts = [hd, c["x"], c["w_router"], np.asarray(c["b_router"], np.float32), c["w1"], c["w2"]]
    if s:
        parts.append(s["emb"])
        for l in range(n_layers):
            parts += [s["w_cat"][l], np.asarray(s["b_f"][l], np.float32), np.asarray(s["b_r"][l], np.float32)]
        parts += [s["w_head"], np.asarray(s["b_head"], np.float32)]
    else:
        parts += [np.zeros(0, c["x"].dtype)] * 2 + [np.zeros(0, np.float32)]
    fin, fout = str(tmp_path / "case.bin"), str(tmp_path / "result.bin")
    with open(fin, "wb") as f:
        for a in parts:
            f.write(np.ascontiguousarray(a).tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([driver, fin, fout], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stderr[-3000:]
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]
    raw = open(fout, "rb").read()
    pos = [0]

    def take(n, dt):
        a = np.frombuffer(raw, dt, n, pos[0])
        pos[0] += a.nbytes
        return a

    edt = c["x"].dtype
    got = dict(idx=take(T, np.int32), prob=take(T, np.float32), counts=take(E, np.int32), replicas=take(E, np.int32),
               slot_base=take(E + 1, np.int32), slot_expert=take(E + R, np.int32), n_slots=int(take(1, np.int32)[0]),
               kept=take(E, np.int32), expert_offset=take(E + 1, np.int32), slot_offset=take(E + R + 1, np.int32),
               perm=take(T, np.int32), inv=take(T, np.int32), h=take(T * F, edt).reshape(T, F),
               y_perm=take(T * d, edt).reshape(T, d), out=take(T * d, edt).reshape(T, d))
    if s:
        got["pred"] = take(s["B"] * s["L"], np.int32)
        got["sru_h"] = take(s["B"] * s["L"] * s["n_hidden"], edt).reshape(-1, s["n_hidden"])
    assert pos[0] == len(raw)
    return got


def _compare(got, c, s, C_, R, policy, residual):
    E = c["E"]
    ref = oracle.layer(c["x"], c["w_router"], c["b_router"], c["w1"], c["w2"], C_, R, policy=policy, residual=residual)
    assert (got["idx"] == ref["route"]["idx"]).all() and (got["prob"] == ref["route"]["prob"]).all()
    for k in ("counts", "replicas", "slot_base", "slot_expert"):
        assert (got[k] == ref["plan"][k]).all(), k
    assert got["n_slots"] == ref["plan"]["n_slots"]
    for k in ("kept", "expert_offset", "slot_offset", "perm", "inv"):
        assert (got[k] == ref["dispatch"][k]).all(), k
    K = int(ref["dispatch"]["expert_offset"][E])
    _, ref_h = oracle.ffn(ref["dispatch"]["x_perm"], c["w1"], c["w2"], ref["dispatch"]["slot_offset"],
                          ref["plan"]["slot_expert"], ref["plan"]["n_slots"], want_h=True)
    assert (got["h"][:K] == ref_h[:K]).all()
    assert (got["y_perm"][:K] == ref["y_perm"][:K]).all()
    assert (got["out"] == ref["out"]).all()
    if s:
        rs = oracle.sru(s["emb"], s["w_cat"], s["b_f"], s["b_r"], s["w_head"], s["b_head"])
        assert (got["pred"] == rs["pred"]).all() and (got["sru_h"] == rs["h"]).all()
    return K


@pytest.mark.parametrize("dtype,T,d,F,E,C_,R,policy,residual", [
    (synth.F32, 97, 16, 24, 5, 9, 3, 0, 0),        # drops and replicas, odd sizes
    (synth.BF16, 130, 24, 40, 7, 6, 4, 1, 1),      # bf16 storage, equal-share policy, residual
    (synth.F32, 3, 8, 8, 6, 1, 0, 0, 0),           # more experts than tokens, no budget
    (synth.BF16, 64, 8, 16, 2, 1, 70, 0, 1),       # slot capacity 1 (the algorithm as printed), budget above the wants
])
def test_layer_and_predictor_under_sanitizers(driver, tmp_path, dtype, T, d, F, E, C_, R, policy, residual):
    c = synth.moe_layer_inputs(T, d, F, E, dtype, 1.2, 300 + T)
    s = synth.sru_inputs(2, 9, 24, 16, 2, E + 3, dtype, 310 + T, bias_std=0.2, w_std=0.2)
    got = _run(driver, tmp_path, c, s, C_, R, policy, residual)
    K = _compare(got, c, s, C_, R, policy, residual)
    assert 0 < K <= T


def test_empty_batch_under_sanitizers(driver, tmp_path):
    c = synth.moe_layer_inputs(4, 8, 8, 3, synth.F32, 1.0, 1)
    c = dict(c, T=0, x=c["x"][:0])
    got = _run(driver, tmp_path, c, None, 2, 2, 0, 0)
    ref_pl = oracle.plan(np.zeros(0, np.int32), 3, 2, 2)
    assert (got["replicas"] == ref_pl["replicas"]).all() and got["n_slots"] == 3
    assert (got["slot_offset"] == 0).all() and (got["kept"] == 0).all()
