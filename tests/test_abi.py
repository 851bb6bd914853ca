"""The C-ABI library loads without a GPU, exports every symbol the header declares, and
rejects bad arguments on the host before anything is launched."""
import ctypes as C
import os
import re

import pytest

import paper_2605_11537_amd as moe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "moe_mpmc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+char\s*\*|int|size_t)\s*\**\s*(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_every_declared_symbol_is_exported():
    L = moe.lib()
    declared = _declared()
    assert set(declared) == set(moe.EXPORTS), (declared, moe.EXPORTS)
    for n in declared:
        assert getattr(L, n) is not None


def test_version_and_error_text():
    L = moe.lib()
    assert L.moe_version() >= 100
    assert isinstance(L.moe_last_error(), bytes)


def test_workspace_queries():
    L = moe.lib()
    assert L.moe_route_workspace_bytes(4096, 768, 128, moe.MOE_BF16) >= 768 * 128 * 2
    assert L.moe_dispatch_workspace_bytes(4096, 128) >= 4 * 128 * 4
    assert L.moe_dispatch_workspace_bytes(-1, 128) == 0
    assert L.moe_packed_weights_bytes(128, 768, 3072, moe.MOE_BF16) == 128 * 768 * 3072 * 2
    assert L.moe_expert_ffn_workspace_bytes(4096, 144, 768, 3072, moe.MOE_BF16) >= 4096 * 3072 * 2


def test_invalid_arguments_are_rejected_on_the_host():
    L = moe.lib()
    buf = (C.c_char * 4096)()
    p = C.cast(buf, C.c_void_p)
    INV, UNS, WS = -1, -2, -3
    q = C.cast(C.addressof(buf) + 1024, C.c_void_p)
    # moe_route
    assert L.moe_route(p, p, 0, None, -1, 64, 8, 0, p, p, None, p, 4096, None) == INV
    assert L.moe_route(p, p, 0, None, 4, 60, 8, 0, p, p, None, p, 4096, None) == INV       # d % 8
    assert L.moe_route(None, p, 0, None, 4, 64, 8, 0, p, p, None, p, 4096, None) == INV
    assert L.moe_route(p, p, 0, None, 4, 64, 8, 7, p, p, None, p, 4096, None) == INV       # dtype
    assert L.moe_route(p, p, 2, None, 4, 64, 8, 0, p, p, None, p, 4096, None) == INV       # layout
    assert L.moe_route(p, p, 1, None, 4, 64, 8, 0, p, p, None, p, 4096, None) == UNS       # packed fp32
    assert L.moe_route(p, p, 0, None, 4, 64, 2048, 0, p, p, None, p, 4096, None) == UNS
    assert L.moe_route(p, p, 0, None, 4, 768, 128, 1, p, p, None, p, 16, None) == WS
    assert b"workspace" in L.moe_last_error()
    # replica_plan
    assert L.replica_plan(p, 4, 8, -1, 1, 0, p, p, p, p, p, None, 0, None) == INV
    assert L.replica_plan(p, 4, 8, 2, 0, 0, p, p, p, p, p, None, 0, None) == INV
    assert L.replica_plan(p, 4, 8, 2, 1, 3, p, p, p, p, p, None, 0, None) == INV
    assert L.replica_plan(p, 4, 4096, 2, 1, 0, p, p, p, p, p, None, 0, None) == UNS
    assert L.replica_plan(p, 65536, 256, 2, 1, 0, p, p, p, p, p, None, 0, None) == WS
    assert L.replica_plan_workspace_bytes(4096, 128) == 0
    assert L.replica_plan_workspace_bytes(65536, 256) >= 8 * 256 * 4
    # moe_dispatch
    assert L.moe_dispatch(p, p, None, 4, 64, 8, 0, 8, 0, p, p, p, p, p, p, p, p, 4096, None) == INV  # C = 0
    assert L.moe_dispatch(p, p, None, 4, 6, 8, 1, 8, 0, p, p, p, p, p, p, p, p, 4096, None) == INV   # row bytes
    assert L.moe_dispatch(p, p, None, 4, 64, 8, 1, 4, 0, p, p, p, p, p, p, p, p, 4096, None) == INV  # max_slots < E
    assert L.moe_dispatch(p, p, None, 4, 64, 8, 1, 8, 0, p, p, p, p, p, p, p, None, 0, None) == WS
    # moe_pack_weights / moe_expert_ffn
    assert L.moe_pack_weights(p, 2, 12, 32, 1, q, None) == INV                       # K % 8
    assert L.moe_pack_weights(p, 2, 16, 16, 1, q, None) == INV                       # N % 32
    assert L.moe_pack_weights(p, 2, 16, 32, 1, p, None) == INV                       # aliasing
    assert L.moe_pack_weights(p, 2, 16, 16, 0, p, None) == UNS
    assert L.moe_expert_ffn(p, None, p, p, 0, p, p, p, 4, 8, 8, 768, 3072, 1, 0, p, p, 1 << 30, None) == UNS  # plain bf16
    assert L.moe_expert_ffn(p, None, p, p, 1, p, p, p, 4, 8, 8, 100, 3072, 1, 0, p, p, 1 << 30, None) == UNS  # d % 128
    assert L.moe_expert_ffn(p, None, p, p, 0, p, p, p, 4, 8, 8, 64, 256, 0, 5, p, p, 1 << 30, None) == INV   # schedule
    assert L.moe_expert_ffn(p, None, p, p, 0, p, p, p, 4, 8, 8, 64, 256, 0, 0, p, p, 16, None) == WS
    # moe_combine
    assert L.moe_combine(p, p, p, p, 4, 64, 0, 2, p, None) == INV                     # residual flag
    assert L.moe_combine(p, q, p, p, 4, 64, 0, 0, q, None) == INV                     # out aliases x
    # top-k entries
    assert L.moe_route_topk(p, p, 0, None, 4, 64, 8, 0, 0, 0, p, p, None, p, 4096, None) == INV    # k = 0
    assert L.moe_route_topk(p, p, 0, None, 4, 64, 8, 0, 9, 0, p, p, None, p, 4096, None) == INV    # k > MOE_MAX_TOPK
    assert L.moe_route_topk(p, p, 0, None, 4, 64, 2, 0, 3, 0, p, p, None, p, 4096, None) == INV    # k > E
    assert L.moe_route_topk(p, p, 0, None, 4, 64, 8, 0, 3, 2, p, p, None, p, 4096, None) == INV    # renormalize flag
    assert L.moe_route_topk(p, p, 0, None, 4, 768, 128, 1, 3, 0, p, p, None, p, 16, None) == WS
    assert L.moe_dispatch_topk(p, p, None, 4, 0, 64, 8, 1, 8, 0, p, p, p, p, p, p, p, p, p, 4096, None) == INV
    assert L.moe_dispatch_topk(p, p, None, 1 << 30, 3, 64, 8, 1, 8, 0, p, p, p, p, p, p, p, p, p, 4096, None) == INV
    assert L.moe_dispatch_topk(p, p, None, 4, 3, 64, 8, 1, 8, 0, p, p, p, p, p, p, None, p, p, 4096, None) == INV
    assert L.moe_dispatch_topk(p, p, None, 4, 3, 64, 8, 1, 8, 0, p, p, p, p, p, p, p, p, None, 0, None) == WS
    assert L.moe_expert_ffn_rows(p, 4, None, p, p, 0, p, p, p, 12, 8, 8, 64, 256, 0, 0, p, p, 1 << 30, None) == INV
    assert L.moe_expert_ffn_rows(p, 0, p, p, p, 0, p, p, p, 12, 8, 8, 64, 256, 0, 0, p, p, 1 << 30, None) == INV
    assert L.moe_expert_ffn_rows(p, 4, p, p, p, 0, p, p, p, 12, 8, 8, 64, 256, 0, 0, p, p, 16, None) == WS
    assert L.moe_combine_topk(p, p, p, p, 4, 9, 64, 0, 0, p, None) == INV              # k
    assert L.moe_combine_topk(p, q, p, p, 4, 3, 64, 0, 0, q, None) == INV              # out aliases x
    assert L.moe_combine_topk(p, p, p, p, 4, 3, 6, 0, 0, p, None) == INV               # row bytes
    # moe_plan_dispatch
    pd = lambda *a: L.moe_plan_dispatch(*a)
    tabs = [p] * 12
    assert pd(p, 4, p, 4, 1, 8, -1, 1, 0, *tabs, None, 0, None) == INV               # budget
    assert pd(p, 4, p, 4, 0, 8, 2, 1, 0, *tabs, None, 0, None) == INV                # k
    assert pd(p, 4, p, 4, 1, 8, 2, 1, 5, *tabs, None, 0, None) == INV                # policy
    assert pd(p, 4, p, 4, 3, 8, 2, 1, 0, *([p] * 11), None, None, 0, None) == INV    # k > 1 without row_token
    assert pd(p, 4, p, 4, 1, 4096, 2, 1, 0, *tabs, None, 0, None) == UNS
    assert pd(p, 100000, p, 100000, 1, 8, 2, 1, 0, *tabs, None, 0, None) == WS
    assert L.moe_plan_dispatch_workspace_bytes(4096, 4096, 1, 128) == 0
    assert L.moe_plan_dispatch_workspace_bytes(4096, 4096, 3, 128) > 0
    # sru_predict
    w = moe.binding.SruWeightsC(2, 768, 256, 128, 0, None, None, None, None, None, 0)
    assert L.sru_predict(p, C.byref(w), 8, 512, 0, p, None, p, 4096, None) == UNS   # fp32 not built
    assert L.sru_predict(p, C.byref(w), 8, 512, 1, p, None, p, 4096, None) == INV   # null tables
    assert L.sru_predict_workspace_bytes(C.byref(w), 8, 512, 1) > 8 * 512 * 1024 * 4
    wa = moe.binding.SruWeightsC(2, 768, 256, 128, 0, None, None, None, None, None, 1)
    assert L.sru_predict(p, C.byref(wa), 8, 2048, 1, p, None, p, 1 << 30, None) == UNS  # attention: L too long
    wa.attention = 3
    assert L.sru_predict(p, C.byref(wa), 8, 512, 1, p, None, p, 1 << 30, None) == INV


def test_new_entry_points_reject_bad_arguments_on_the_host():
    L = moe.lib()
    buf = (C.c_char * 4096)()
    p = C.cast(buf, C.c_void_p)
    INV, UNS = -1, -2
    # moe_dispatch_static: the checks of moe_dispatch, and its own size limit (refused before any device call)
    ds = L.moe_dispatch_static
    assert ds(p, p, None, 4, 64, 8, 0, 8, 0, p, p, p, p, p, p, p, None) == INV            # C = 0
    assert ds(p, p, None, 4, 6, 8, 1, 8, 0, p, p, p, p, p, p, p, None) == INV             # row bytes
    assert ds(p, p, None, 4, 64, 8, 1, 4, 0, p, p, p, p, p, p, p, None) == INV            # max_slots < E
    assert ds(p, p, None, 300000, 64, 1024, 1, 1024, 0, p, p, p, p, p, p, p, None) == UNS  # 293 blocks x 1024 experts
    assert b"static scratch" in L.moe_last_error()
    # moe_expert_ffn_timed: same validation as the untimed calls
    ft = L.moe_expert_ffn_timed
    assert ft(p, 4, None, p, p, 0, p, p, p, 12, 8, 8, 64, 256, 0, 0, p, p, 1 << 30, None, None, None, None) == INV  # n_x_rows != max_rows
    assert ft(p, 4, None, p, p, 0, p, p, p, 4, 8, 8, 64, 256, 0, 5, p, p, 1 << 30, None, None, None, None) == INV   # schedule
    assert ft(p, 4, None, p, p, 0, p, p, p, 4, 8, 8, 768, 3072, 1, 0, p, p, 1 << 30, None, None, None, None) == UNS  # plain bf16
    # measurement calls
    assert L.moe_measure_stream_read(None, 1 << 20, 0, 0, p, None) == INV
    assert L.moe_measure_stream_read(p, 100, 0, 0, p, None) == INV                        # not a multiple of 16
    assert L.moe_measure_stream_read(p, 1 << 20, 2, 0, p, None) == INV                    # flag
    assert L.moe_measure_mfma_bf16(0, 0, p, None) == INV
    assert L.moe_measure_mfma_bf16(10, 2, p, None) == INV
    assert L.moe_measure_mfma_bf16_flops(0) == 0
    assert L.moe_build_id() is not None


def test_a_library_built_from_other_sources_is_refused(monkeypatch):
    """binding.lib() compares the source hash compiled into the library with the sources beside it."""
    from paper_2605_11537_amd import binding, build
    L = moe.lib()
    L.moe_build_id.restype = C.c_char_p
    assert L.moe_build_id().decode() == build.source_id()
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(build, "source_id", lambda: "0123456789abcdef")
    with pytest.raises(RuntimeError) as ei:
        binding.lib()
    assert "rebuild" in str(ei.value)
    monkeypatch.undo()
    assert binding.lib() is not None


def test_bench_refuses_more_than_one_gpu():
    """One GPU per box: the bench says so and exits before touching any device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""
