"""GPU parity of hikonv_conv2d_fused (one kernel per layer: convolution, ReLU, requantisation,
optional 2x2 max-pool, packing for the next layer) through the C ABI against the oracle chain
direct convolution -> relu_requant -> maxpool -> direct convolution, bit-exact: both this
layer's accumulators and the next layer's result computed from the packed words it wrote."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import direct

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_00763_amd as hk
    from gpu_util import dnn_plan, dev, compact, Guarded

CASES = [  # n, c, h, w, co, k, pad, pool, shift | next: co2, k2, pad2
    (1, 3, 8, 12, 16, 3, 1, 1, 3, 8, 3, 1),
    (2, 5, 9, 17, 9, 3, 1, 1, 4, 5, 3, 1),          # odd sizes: the last row and column are dropped by the pool
    (1, 16, 6, 40, 32, 3, 1, 0, 5, 8, 3, 1),
    (2, 8, 5, 7, 12, 3, 0, 0, 2, 4, 1, 0),          # no padding, 1x1 follower
    (1, 4, 4, 150, 8, 3, 1, 1, 3, 8, 3, 1),         # rows longer than a wave: 63-block segments
    (1, 3, 6, 320, 16, 3, 1, 1, 4, 8, 3, 1),        # the first layer of the 4-bit network at full width
    (3, 64, 10, 20, 64, 3, 1, 0, 7, 36, 1, 0),      # eight channel tiles, three images, term range over eight waves
    (1, 64, 4, 9, 36, 1, 0, 0, 3, 6, 3, 1),         # 36 channels: the last tile is half empty; 1x1 kernel
    (2, 12, 7, 30, 13, 3, 1, 1, 3, 7, 3, 1),        # 13 channels: a quad of the next layer padded with zero words
    (2, 8, 23, 5, 8, 3, 1, 1, 2, 8, 3, 1),          # short rows: many rows per wave, odd row count with pooling
    (1, 8, 40, 14, 16, 3, 1, 0, 3, 8, 3, 1),        # four rows per wave, no pooling
    (4, 4, 3, 9, 8, 3, 1, 1, 2, 4, 3, 1),           # three rows in all: one pooled row, the third row dropped
    (1, 256, 6, 12, 8, 3, 1, 0, 8, 8, 1, 0),        # 768 terms: the packed input of a workgroup exceeds its LDS
    (1, 7, 2, 9, 3, 1, 0, 1, 0, 2, 3, 1),           # one workgroup per image writes both padding rows
    (1, 6, 1, 9, 8, 3, 1, 0, 1, 8, 3, 1),           # a single output row
]


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("tight", [0, 1])
def test_fused_layer_matches_oracle_chain(case, tight):
    n, c, h, w, co, k, pad, pool, shift, co2, k2, pad2 = case
    rng = wl.rng_for("fused", case)
    x = wl.uniform_values(rng, (n, c, h, w), 4, False)
    w1 = wl.uniform_values(rng, (co, c, k, k), 4, True)
    w2 = wl.uniform_values(rng, (co2, co, k2, k2), 4, True)
    ref1 = direct.conv2d(x, w1, 1, pad)
    q = direct.relu_requant(ref1, shift, 15)
    if pool:
        q = direct.maxpool2x2(q)
    hn, wn = q.shape[2], q.shape[3]
    ref2 = direct.conv2d(q.view(np.uint8), w2, 1, pad2)
    ho, wo = ref1.shape[2], ref1.shape[3]
    plan1 = dnn_plan(4, 4, False, True, k, 0, tight=tight)
    plan2 = dnn_plan(4, 4, False, True, k2, 0, tight=tight)
    ws1 = Guarded(hk.hikonv_conv2d_workspace_bytes(plan1, n, c, h, w, co, k, k, 1, pad, True), torch.uint8, 0x5A)
    ws2 = Guarded(hk.hikonv_conv2d_workspace_bytes(plan2, n, co, hn, wn, co2, k2, k2, 1, pad2, True), torch.uint8, 0x5A)
    pw1 = torch.empty(hk.hikonv_packed_weights_bytes(plan1, co, c, k, k), dtype=torch.uint8, device="cuda")
    pw2 = torch.empty(hk.hikonv_packed_weights_bytes(plan2, co2, co, k2, k2), dtype=torch.uint8, device="cuda")
    hk.hikonv_pack_weights(plan1, dev(w1), co, c, k, k, pw1)
    hk.hikonv_pack_weights(plan2, dev(w2), co2, co, k2, k2, pw2)
    for keep_y in (True, False):
        y1 = Guarded(ref1.size)
        y2 = Guarded(ref2.size)
        ws2.view.fill_(0x5A)
        x_bd = compact(x.reshape(n * c * h, w), 4)
        # bit-dense input with a workspace, one value per byte without one (the workgroups pack
        # their own input rows whenever those fit their LDS, which holds for every case here but the widest)
        if keep_y:
            hk.hikonv_conv2d_fused(plan1, x_bd, hk.FMT_BITDENSE, n, c, h, w, pw1, co, k, k, pad, ws1.view, y1.view, shift,
                                   15, bool(pool), plan2, co2, k2, k2, pad2, ws2.view)
        else:
            own = hk.with_fields(plan1, kernel=hk.KERNEL_LDS)   # the workgroups pack their own input rows
            try:
                hk.hikonv_conv2d_fused(own, dev(x), hk.FMT_INT8, n, c, h, w, pw1, co, k, k, pad, None, None, shift, 15,
                                       bool(pool), plan2, co2, k2, k2, pad2, ws2.view)
            except hk.HikonvError as err:
                assert err.code == hk.EWORKSPACE          # too large for in-kernel packing: the workspace is needed
                hk.hikonv_conv2d_fused(own, dev(x), hk.FMT_INT8, n, c, h, w, pw1, co, k, k, pad, ws1.view, None, shift,
                                       15, bool(pool), plan2, co2, k2, k2, pad2, ws2.view)
        # the follower reads the packed words the first kernel wrote; as a plain layer through the same entry point
        hk.hikonv_conv2d_fused(plan2, None, hk.FMT_PACKED, n, co, hn, wn, pw2, co2, k2, k2, pad2, ws2.view, y2.view)
        got2 = y2.result().reshape(ref2.shape)
        got1 = y1.result().reshape(ref1.shape)
        ws1.check()
        ws2.check()
        if keep_y:
            assert np.array_equal(got1, ref1), case
        else:
            assert (got1 == -77777).all(), "accumulators stored although y was not asked for"
        assert np.array_equal(got2, ref2), case
        # and through the two-kernel form on the same packed words
        y3 = Guarded(ref2.size)
        hk.hikonv_conv2d_prepacked(plan2, None, hk.FMT_PACKED, n, co, hn, wn, pw2, co2, k2, k2, 1, pad2, ws2.view, y3.view)
        assert np.array_equal(y3.result().reshape(ref2.shape), ref2), case
    assert ho == h + 2 * pad - k + 1 and wo == w + 2 * pad - k + 1


def test_fused_layer_extreme_values_and_clamp():
    """All-maximum activations against all-minimum and all-maximum weights: the largest sums the
    plan admits; shifts that clamp everything or nothing."""
    n, c, h, w, co = 1, 24, 6, 11, 8
    plan = dnn_plan(4, 4, False, True, 3, 0)
    for wv in (-8, 7):
        x = np.full((n, c, h, w), 15, dtype=np.uint8)
        w1 = np.full((co, c, 3, 3), wv, dtype=np.int8)
        w2 = wl.uniform_values(wl.rng_for("fx", wv), (4, co, 3, 3), 4, True)
        ref1 = direct.conv2d(x, w1, 1, 1)
        for shift in (0, 4, 9):
            qq = direct.maxpool2x2(direct.relu_requant(ref1, shift, 15))
            ref2 = direct.conv2d(qq.view(np.uint8), w2, 1, 1)
            ws1 = torch.empty(hk.hikonv_conv2d_workspace_bytes(plan, n, c, h, w, co, 3, 3, 1, 1, True), dtype=torch.uint8, device="cuda")
            ws2 = torch.empty(hk.hikonv_conv2d_workspace_bytes(plan, n, co, 3, 5, 4, 3, 3, 1, 1, True), dtype=torch.uint8, device="cuda")
            pw1 = torch.empty(hk.hikonv_packed_weights_bytes(plan, co, c, 3, 3), dtype=torch.uint8, device="cuda")
            pw2 = torch.empty(hk.hikonv_packed_weights_bytes(plan, 4, co, 3, 3), dtype=torch.uint8, device="cuda")
            hk.hikonv_pack_weights(plan, dev(w1), co, c, 3, 3, pw1)
            hk.hikonv_pack_weights(plan, dev(w2), 4, co, 3, 3, pw2)
            y1, y2 = Guarded(ref1.size), Guarded(ref2.size)
            hk.hikonv_conv2d_fused(plan, dev(x), hk.FMT_INT8, n, c, h, w, pw1, co, 3, 3, 1, ws1, y1.view, shift, 15, True,
                                   plan, 4, 3, 3, 1, ws2)
            hk.hikonv_conv2d_fused(plan, None, hk.FMT_PACKED, n, co, 3, 5, pw2, 4, 3, 3, 1, ws2, y2.view)
            assert np.array_equal(y1.result().reshape(ref1.shape), ref1), (wv, shift)
            assert np.array_equal(y2.result().reshape(ref2.shape), ref2), (wv, shift)


def test_fused_layer_refusals():
    plan = dnn_plan(4, 4, False, True, 3, 0)
    x = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    big = torch.zeros(1 << 22, dtype=torch.uint8, device="cuda")
    y = torch.zeros(1 << 16, dtype=torch.int32, device="cuda")
    # rows of 1600 values: two rows of nine 63-block segments are more waves than a workgroup holds
    with pytest.raises(hk.HikonvError) as e:
        hk.hikonv_conv2d_fused(plan, x, hk.FMT_INT8, 1, 1, 2, 1600, big, 8, 3, 3, 1, big, y, 0, 15, True, plan, 8, 3, 3, 1, big)
    assert e.value.code == hk.EUNSUPPORTED
    # 2048 channels: the tile's weight words (6144 terms x 32 bytes) do not fit the workgroup's LDS
    with pytest.raises(hk.HikonvError) as e:
        hk.hikonv_conv2d_fused(plan, x, hk.FMT_PACKED, 1, 2048, 4, 8, big, 8, 3, 3, 1, big, y)
    assert e.value.code == hk.EUNSUPPORTED
    # neither accumulators nor a follower asked for
    with pytest.raises(hk.HikonvError) as e:
        hk.hikonv_conv2d_fused(plan, x, hk.FMT_INT8, 1, 1, 4, 8, big, 8, 3, 3, 1, big, None)
    assert e.value.code == hk.EINVAL
    # a follower with signed activations; qmax beyond its width; its workspace too small
    signed_next = dnn_plan(4, 4, True, True, 3, 0)
    for kwargs, code in ((dict(next_plan=signed_next), hk.EUNSUPPORTED), (dict(qmax=16), hk.EINVAL),
                         (dict(nws=big[:256]), hk.EWORKSPACE), (dict(shift=32), hk.EINVAL)):
        a = dict(next_plan=plan, qmax=15, nws=big, shift=0)
        a.update(kwargs)
        with pytest.raises(hk.HikonvError) as e:
            hk.hikonv_conv2d_fused(plan, x, hk.FMT_INT8, 1, 1, 4, 8, big, 8, 3, 3, 1, big, y, a["shift"], a["qmax"], False,
                                   a["next_plan"], 8, 3, 3, 1, a["nws"])
        assert e.value.code == code, kwargs
    # plans with more than four slices per word are left to the two-kernel form
    wide_n = dnn_plan(1, 1, False, False, 3, 0, bipolar=False)
    if wide_n.N > 4:
        with pytest.raises(hk.HikonvError) as e:
            hk.hikonv_conv2d_fused(wide_n, x, hk.FMT_INT8, 1, 1, 4, 8, big, 8, 3, 3, 1, big, y)
        assert e.value.code == hk.EUNSUPPORTED
    torch.cuda.synchronize()
