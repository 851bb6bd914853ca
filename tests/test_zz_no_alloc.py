"""moe_dispatch_static (the allocation-free variant: block histograms in the library's static device
array) against moe_dispatch on the same inputs, bit for bit, through the C ABI: two calls in a row,
the second on a smaller batch (so stale entries of the first call sit in the shared array), then a
larger one again, and the size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth
from gpu_util import to_dev

pytestmark = pytest.mark.gpu

KEYS = ("counts", "kept", "expert_offset", "slot_offset", "perm", "inv")


def _buffers(T, d, E, max_slots, dtype):
    i32 = lambda n: torch.full((n,), -7, dtype=torch.int32, device="cuda")
    return dict(counts=i32(E), kept=i32(E), expert_offset=i32(E + 1), slot_offset=i32(max_slots + 1), perm=i32(T),
                inv=i32(T), x_perm=torch.zeros(T, d, dtype=dtype, device="cuda"))


def _case(moe, T, d, E, C_, R, seed):
    rng = np.random.default_rng(seed)
    ids = to_dev(rng.choice(E, size=T, p=rng.dirichlet(np.ones(E) * 0.3)).astype(np.int32))
    x = to_dev(synth.normal_tensor((T, d), 1.0, [seed, T], synth.BF16))
    rep = moe.replica_plan(ids, E, R, C_)["replicas"]
    return ids, x, rep


def test_dispatch_static_equals_dispatch_two_calls_in_a_row():
    import paper_2605_11537_amd as moe
    L = moe.lib()
    # larger batch first (70 token blocks x 300 experts), then a smaller one with fewer experts, then large again
    for T, d, E, C_, R, seed in [(70001, 32, 300, 150, 64, 1), (3001, 64, 24, 90, 5, 2), (16384, 128, 256, 64, 32, 3)]:
        ids, x, rep = _case(moe, T, d, E, C_, R, seed)
        ref = moe.moe_dispatch(x, ids, rep, E, C_, E + R)
        got = _buffers(T, d, E, E + R, torch.bfloat16)
        before = torch.cuda.memory_allocated()
        rc = L.moe_dispatch_static(C.c_void_p(x.data_ptr()), C.c_void_p(ids.data_ptr()), C.c_void_p(rep.data_ptr()),
                                   T, d, E, C_, E + R, moe.MOE_BF16, *[C.c_void_p(got[k].data_ptr()) for k in KEYS],
                                   C.c_void_p(got["x_perm"].data_ptr()),
                                   C.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0, L.moe_last_error()
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        for k in KEYS:
            assert torch.equal(got[k], ref[k]), (T, k)
        K = int(ref["expert_offset"][E].item())
        assert torch.equal(got["x_perm"][:K], ref["x_perm"][:K]), T
        print(f"dispatch_static T={T} E={E}: kept {K}, tables and rows equal", flush=True)
    # index tables only (no row copy), through the binding
    ids, x, rep = _case(moe, 5000, 72, 100, 9, 20, 4)
    ref = moe.moe_dispatch(None, ids, rep, 100, 9, 120, shape=(5000, 72), dtype=torch.bfloat16)
    got = moe.moe_dispatch_static(None, ids, rep, 100, 9, 120, _buffers(5000, 72, 100, 120, torch.bfloat16),
                                  shape=(5000, 72), dtype=torch.bfloat16)
    for k in KEYS:
        assert torch.equal(got[k], ref[k]), k


def test_dispatch_static_rejects_sizes_beyond_its_array():
    import paper_2605_11537_amd as moe
    L = moe.lib()
    T, E = 300000, 1024                     # 293 blocks x 1024 experts > 262144 entries
    ids = torch.zeros(T, dtype=torch.int32, device="cuda")
    got = _buffers(T, 8, E, E, torch.float32)
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_dispatch_static(None, ids, None, E, 4, E, got, shape=(T, 8), dtype=torch.float32)
    assert ei.value.code == -2 and "static scratch" in str(ei.value)
    assert L.moe_dispatch_static(None, None, None, -1, 8, E, 4, E, 0, None, None, None, None, None, None, None,
                                 None) == -1
