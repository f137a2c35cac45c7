"""GPU check of hikonv_conv2d_noalloc (the layer call for callers that cannot allocate): its
output equals hikonv_conv2d's, and the oracle's, on two calls in a row, the second one on a
smaller layer (so the library's fixed array still holds the first call's words), and a layer
beyond the array's size is refused."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_00763_amd as hk
    from gpu_util import run_conv2d, dnn_plan, dev
    from oracle import direct


def _noalloc(plan, x_np, w_np, stride, pad):
    n, c, h, w = x_np.shape
    co, _, kh, kw = w_np.shape
    ho, wo = (h + 2 * pad - kh) // stride + 1, (w + 2 * pad - kw) // stride + 1
    y = torch.full((64 + n * co * ho * wo + 64,), -77777, dtype=torch.int32, device="cuda")
    hk.hikonv_conv2d_noalloc(plan, dev(x_np), hk.FMT_INT8, n, c, h, w, dev(w_np), co, kh, kw, stride, pad, y[64:])
    torch.cuda.synchronize()
    res = y.cpu().numpy()
    assert (res[:64] == -77777).all() and (res[64 + n * co * ho * wo:] == -77777).all(), "wrote outside the output"
    return res[64:64 + n * co * ho * wo].reshape(n, co, ho, wo)


def test_noalloc_matches_conv2d_twice_second_call_smaller():
    cases = [
        # first a layer that uses a good part of the array, then smaller ones of other shapes and plans
        (dict(bits_a=4, bits_w=4, a_signed=True, w_signed=True), (2, 64, 56, 56), 64, 3, 1, 1),
        (dict(bits_a=4, bits_w=4, a_signed=True, w_signed=True), (1, 16, 20, 33), 24, 3, 1, 1),
        (dict(bits_a=2, bits_w=2, a_signed=False, w_signed=True), (1, 5, 9, 17), 3, 3, 2, 1),
        (dict(bits_a=4, bits_w=4, a_signed=False, w_signed=True), (3, 32, 28, 28), 40, 1, 1, 0),
    ]
    for kw_plan, shape, co, k, stride, pad in cases:
        n, c, h, w = shape
        rng = wl.rng_for("noalloc", shape, co, k)
        x = wl.uniform_values(rng, shape, kw_plan["bits_a"], kw_plan["a_signed"])
        wt = wl.uniform_values(rng, (co, c, k, k), kw_plan["bits_w"], kw_plan["w_signed"])
        plan = dnn_plan(kw_plan["bits_a"], kw_plan["bits_w"], kw_plan["a_signed"], kw_plan["w_signed"], k, 0)
        need = hk.hikonv_conv2d_workspace_bytes(plan, n, c, h, w, co, k, k, stride, pad, False)
        assert 0 < need <= hk.NOALLOC_SCRATCH_BYTES
        got = _noalloc(plan, x, wt, stride, pad)
        assert np.array_equal(got, run_conv2d(plan, x, wt, stride, pad)), shape
        assert np.array_equal(got, direct.conv2d(x, wt, stride, pad)), shape


def test_noalloc_rejects_layers_beyond_the_fixed_array():
    plan = dnn_plan(4, 4, True, True, 3, 0)
    n, c, h, w, co = 64, 64, 56, 56, 64
    assert hk.hikonv_conv2d_workspace_bytes(plan, n, c, h, w, co, 3, 3, 1, 1, False) > hk.NOALLOC_SCRATCH_BYTES
    x = torch.zeros(16, dtype=torch.uint8, device="cuda")          # never read: the call is refused on the host
    with pytest.raises(hk.HikonvError) as e:
        hk.hikonv_conv2d_noalloc(plan, x, hk.FMT_INT8, n, c, h, w, x, co, 3, 3, 1, 1, x)
    assert e.value.code == hk.ESCRATCH
    with pytest.raises(hk.HikonvError) as e:
        hk.hikonv_conv2d_noalloc(plan, x, hk.FMT_PACKED, 1, 4, 8, 8, x, 8, 3, 3, 1, 1, x)
    assert e.value.code == hk.EINVAL
    torch.cuda.synchronize()
