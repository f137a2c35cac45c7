"""GPU parity of the two widened layer forms: column stride as a sum over packed column
phases (polyphase) and the three-dimensional layer, through the C ABI vs the int64 oracle,
bit-exact.  Every case also runs with the scalar-register kernel forced."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import direct

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_00763_amd as hk
    import gpu_util
    from gpu_util import run_conv2d, run_conv3d, dnn_plan


@pytest.fixture(params=["default", "scalar_register_kernel"])
def kernel_choice(request):
    old = dict(gpu_util.LAYER_DEFAULTS)
    if request.param == "scalar_register_kernel":
        gpu_util.LAYER_DEFAULTS.update(kernel=hk.KERNEL_SREG)
    yield request.param
    gpu_util.LAYER_DEFAULTS.update(old)


def _values(tag, bits, a_s, w_s, xshape, wshape):
    rng = wl.rng_for(tag, bits, a_s, w_s, xshape, wshape)
    return wl.uniform_values(rng, xshape, bits, a_s), wl.uniform_values(rng, wshape, bits, w_s)


def _plans(bits, a_s, w_s, kw, stride, wide=True):
    """(label, plan) for the decimating form and, where it differs, the polyphase form."""
    out = []
    taps_poly = -(-kw // stride)
    for label, taps in (("decimate", kw), ("polyphase", taps_poly)):
        if label == "polyphase" and (stride == 1 or taps == kw):
            continue
        for m in (0, 5):
            try:
                plan = dnn_plan(bits, bits, a_s, w_s, taps, m, wide)
            except hk.HikonvError as e:
                assert e.code == hk.ENOPLAN
                continue
            assert plan.N <= hk.LAYER_MAX_N
            out.append((label, plan))
    return out


STRIDED = [  # n, c, h, w, co, kh, kw, stride, pad
    (1, 3, 9, 17, 8, 3, 3, 2, 1),
    (2, 5, 8, 16, 9, 3, 3, 2, 0),
    (1, 4, 11, 23, 4, 5, 5, 2, 2),
    (1, 6, 10, 31, 12, 3, 7, 2, 3),
    (1, 2, 12, 40, 8, 3, 5, 3, 1),
    (1, 7, 9, 29, 10, 2, 4, 4, 0),
    (1, 3, 7, 300, 8, 3, 3, 2, 1),     # long rows
    (1, 3, 8, 19, 16, 3, 7, 2, 5),     # padding wider than the polyphase kernel
    (1, 20, 14, 14, 24, 3, 3, 2, 1),   # enough terms to divide them over the waves of a workgroup
]


@pytest.mark.parametrize("bits,signs", [(1, (False, False)), (2, (True, True)), (4, (True, True)), (4, (False, True)),
                                        (8, (False, False)), (3, (False, True))])
def test_polyphase_stride_matches_oracle(bits, signs, kernel_choice):
    a_s, w_s = signs
    ran = {"decimate": 0, "polyphase": 0}
    for shape in STRIDED:
        n, c, h, w, co, kh, kw, stride, pad = shape
        x, wt = _values("p1", bits, a_s, w_s, (n, c, h, w), (co, c, kh, kw))
        ref = direct.conv2d(x, wt, stride, pad)
        for label, plan in _plans(bits, a_s, w_s, kw, stride):
            if label == "decimate" and pad > kw - 1:
                continue
            for fmt, pre in ((hk.FMT_INT8, False), (hk.FMT_BITDENSE, True)):
                got = run_conv2d(plan, x, wt, stride, pad, fmt, prepacked=pre)
                assert np.array_equal(got, ref), (shape, label, fmt, plan)
                ran[label] += 1
    assert ran["polyphase"] > 0 and ran["decimate"] > 0


def test_polyphase_stride_narrow_multiplier():
    for shape in STRIDED[:5]:
        n, c, h, w, co, kh, kw, stride, pad = shape
        x, wt = _values("p2", 2, False, True, (n, c, h, w), (co, c, kh, kw))
        ref = direct.conv2d(x, wt, stride, pad)
        for label, plan in _plans(2, False, True, kw, stride, wide=False):
            if label == "decimate" and pad > kw - 1:
                continue
            assert np.array_equal(run_conv2d(plan, x, wt, stride, pad), ref), (shape, label, plan)


def test_polyphase_rejections():
    plan = dnn_plan(4, 4, True, True, 2, 0, True)
    assert hk.hikonv_conv2d_workspace_bytes(plan, 1, 4, 8, 8, 8, 3, 3, 1, 1, False) == 0   # taps fit no form at stride 1
    assert hk.hikonv_conv2d_workspace_bytes(plan, 1, 4, 8, 8, 8, 3, 3, 2, 1, False) > 0


def test_bipolar_layers_in_both_widened_forms(kernel_choice):
    # {-1,+1} values travel as signed slices (0 in the zero padding), so every layer form takes them
    for shape in ((1, 6, 9, 17, 8, 3, 3, 2, 1), (2, 5, 8, 16, 9, 3, 5, 2, 2), (1, 40, 7, 15, 8, 3, 3, 3, 1)):
        n, c, h, w, co, kh, kw, stride, pad = shape
        x, wt = wl.bipolar_case(n, c, h, w, co, kh, kw, tag="p4")
        ref = direct.conv2d(x, wt, stride, pad)
        for taps in (kw, -(-kw // stride)):
            plan = dnn_plan(1, 1, False, False, taps, 0, True, bipolar=True)
            for fmt, pre in ((hk.FMT_INT8, False), (hk.FMT_BITDENSE, True)):
                assert np.array_equal(run_conv2d(plan, x, wt, stride, pad, fmt, prepacked=pre), ref), (shape, taps, fmt, plan)
    rng = wl.rng_for("p5")
    x = (rng.integers(0, 2, (1, 5, 4, 6, 9)) * 2 - 1).astype(np.int8)
    wt = (rng.integers(0, 2, (8, 5, 3, 3, 3)) * 2 - 1).astype(np.int8)
    plan = dnn_plan(1, 1, False, False, 3, 0, True, bipolar=True)
    for fmt, pre in ((hk.FMT_INT8, False), (hk.FMT_BITDENSE, True)):
        # bit-dense {-1,+1} volumes: bit 1 stands for +1
        got = run_conv3d(plan, x, wt, 1, 1, fmt, prepacked=pre)
        assert np.array_equal(got, direct.conv3d(x, wt, 1, 1)), (fmt, plan)


VOLUMES = [  # n, c, d, h, w, co, kd, kh, kw, stride, pad
    (1, 2, 4, 5, 7, 3, 3, 3, 3, 1, 1),
    (2, 3, 5, 6, 9, 8, 3, 3, 3, 1, 0),
    (1, 4, 6, 6, 11, 9, 2, 3, 3, 2, 1),
    (1, 2, 7, 8, 13, 8, 3, 2, 5, 2, 2),
    (1, 5, 3, 4, 70, 4, 1, 3, 3, 1, 1),     # depth-1 kernel, long rows
    (1, 3, 8, 5, 6, 16, 5, 1, 1, 1, 2),     # only the depth axis has extent
    (1, 8, 6, 7, 9, 17, 3, 3, 3, 1, 1),     # enough terms to divide them over the waves of a workgroup
]


@pytest.mark.parametrize("bits,signs", [(1, (False, False)), (2, (True, True)), (4, (True, True)), (4, (False, True)),
                                        (8, (True, True))])
def test_conv3d_matches_oracle(bits, signs, kernel_choice):
    a_s, w_s = signs
    ran = 0
    for shape in VOLUMES:
        n, c, d, h, w, co, kd, kh, kw, stride, pad = shape
        x, wt = _values("v1", bits, a_s, w_s, (n, c, d, h, w), (co, c, kd, kh, kw))
        ref = direct.conv3d(x, wt, stride, pad)
        for label, plan in _plans(bits, a_s, w_s, kw, stride):
            if label == "decimate" and pad > kw - 1:
                continue
            for fmt, pre in ((hk.FMT_INT8, False), (hk.FMT_BITDENSE, True)):
                got = run_conv3d(plan, x, wt, stride, pad, fmt, prepacked=pre)
                assert np.array_equal(got, ref), (shape, label, fmt, plan)
                ran += 1
    assert ran > 0


def test_conv3d_extreme_values_and_2d_special_case():
    for bits, a_s, w_s in ((4, True, True), (4, False, True), (8, True, True)):
        lo_a, hi_a = wl.value_range(bits, a_s)
        lo_w, hi_w = wl.value_range(bits, w_s)
        for av, wv in ((lo_a, lo_w), (lo_a, hi_w), (hi_a, lo_w), (hi_a, hi_w)):
            x = np.full((1, 6, 4, 5, 9), av, dtype=np.int8 if a_s else np.uint8)
            w = np.full((8, 6, 3, 3, 3), wv, dtype=np.int8 if w_s else np.uint8)
            plan = dnn_plan(bits, bits, a_s, w_s, 3, 0, True)
            assert np.array_equal(run_conv3d(plan, x, w, 1, 1), direct.conv3d(x, w, 1, 1)), (bits, av, wv, plan)
    # a volume of depth 1 with a depth-1 kernel is the 2-D layer
    x, wt = _values("v2", 4, True, True, (2, 5, 1, 9, 12), (8, 5, 1, 3, 3))
    plan = dnn_plan(4, 4, True, True, 3, 0, True)
    got3 = run_conv3d(plan, x, wt, 1, 0)
    got2 = run_conv2d(plan, x[:, :, 0], wt[:, :, 0], 1, 0)
    assert np.array_equal(got3[:, :, 0], got2)
