"""Helpers of the GPU parity tests: numpy storage <-> device tensors, tolerances."""
import numpy as np
import torch

import synth


def to_dev(a):
    """numpy array in generator storage (float32 / uint16 bf16 bits / int32) -> cuda tensor."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host(t):
    """cuda tensor -> numpy in generator storage."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def f64(a):
    return synth.storage_to_f64(a)


# tolerances of the benchmark spec: fp32 max abs error 1e-4; bf16 (fp32 accumulate) max relative
# error 2e-2, taken as max|diff| / max|reference| over the tensor
def assert_close(got, ref, dtype, what=""):
    g, r = f64(got), f64(ref)
    assert g.shape == r.shape, (what, g.shape, r.shape)
    if g.size == 0:
        return
    diff = np.abs(g - r).max()
    if dtype == synth.F32:
        assert diff <= 1e-4, f"{what}: max abs error {diff:.3e} > 1e-4"
    else:
        scale = np.abs(r).max()
        assert diff <= 2e-2 * scale, f"{what}: max rel error {diff / max(scale, 1e-30):.3e} > 2e-2"


def check_ids_margin(got, ref_idx, ref_idx2, ref_margin, tau, what=""):
    """Float->int decision: identical wherever the oracle's top-2 gap exceeds tau; inside the
    gap the runner-up is also accepted.  Returns the number of flipped tokens."""
    got = np.asarray(got)
    diff = got != ref_idx
    clear = ref_margin > tau
    assert not (diff & clear).any(), \
        f"{what}: {int((diff & clear).sum())} ids differ where the top-2 gap exceeds {tau:g}"
    assert (got[diff] == ref_idx2[diff]).all(), f"{what}: a near-tie resolved to a third id"
    return int(diff.sum())
