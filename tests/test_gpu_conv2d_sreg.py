"""GPU parity of the layer kernel that keeps the weight words in scalar registers.  The
library picks it by itself only for large layers; here the plans ask for it
(kernel = HIKONV_KERNEL_SREG) wherever the plan allows it, so that small and ragged shapes
reach it too.  Through the
C ABI vs the int64 oracle, bit-exact."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import direct

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_00763_amd as hk
    import gpu_util
    from gpu_util import run_conv2d, dnn_plan


@pytest.fixture(autouse=True)
def force_scalar_register_kernel():
    old = dict(gpu_util.LAYER_DEFAULTS)
    gpu_util.LAYER_DEFAULTS.update(kernel=hk.KERNEL_SREG, flags=0)
    yield
    gpu_util.LAYER_DEFAULTS.update(old)


SHAPES = [  # n, c, h, w, co, kh, kw, stride, pad
    (1, 3, 5, 7, 8, 3, 3, 1, 1),
    (2, 5, 9, 11, 9, 3, 3, 1, 0),
    (1, 4, 8, 8, 16, 1, 1, 1, 0),      # one tap: no high segments
    (1, 6, 10, 13, 12, 3, 3, 2, 1),    # stride 2
    (1, 7, 6, 9, 10, 3, 2, 1, 1),      # two taps: one high segment
    (1, 3, 4, 300, 8, 3, 3, 1, 1),     # rows longer than a wave: segments with a recomputed block
    (1, 24, 6, 9, 17, 3, 3, 1, 2),     # enough terms for the term range to be divided over four waves
    (3, 9, 4, 64, 8, 3, 3, 1, 1),      # row length a multiple of every N
    (1, 2, 7, 20, 8, 5, 5, 1, 2),      # five taps (chunked or wide B words): falls back where the kernel does not apply
]


def _case(bits, a_s, w_s, shape, tag):
    n, c, h, w, co, kh, kw, _, _ = shape
    rng = wl.rng_for(tag, bits, a_s, w_s, shape)
    return wl.uniform_values(rng, (n, c, h, w), bits, a_s), wl.uniform_values(rng, (co, c, kh, kw), bits, w_s)


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 6, 8])
@pytest.mark.parametrize("signs", [(False, False), (True, True), (False, True)])
def test_scalar_register_kernel_small_shapes(bits, signs):
    a_s, w_s = signs
    ran = 0
    for shape in SHAPES:
        x, w = _case(bits, a_s, w_s, shape, "s1")
        stride, pad, kw = shape[7], shape[8], shape[6]
        ref = direct.conv2d(x, w, stride, pad)
        for m in (4, 7, 0):
            for tight in (0, 1):
                try:
                    plan = dnn_plan(bits, bits, a_s, w_s, kw, m, True, tight=tight)
                except hk.HikonvError as e:
                    assert e.code == hk.ENOPLAN
                    continue
                got = run_conv2d(plan, x, w, stride, pad, hk.FMT_BITDENSE, prepacked=(m == 4))
                assert np.array_equal(got, ref), (bits, signs, shape, m, tight, plan)
                ran += 1
    assert ran > 0


def test_scalar_register_kernel_extreme_values():
    for bits, a_s, w_s in ((4, True, True), (4, False, True), (4, False, False), (2, True, True), (8, True, True)):
        lo_a, hi_a = wl.value_range(bits, a_s)
        lo_w, hi_w = wl.value_range(bits, w_s)
        for av in (lo_a, hi_a):
            for wv in (lo_w, hi_w):
                x = np.full((1, 20, 6, 9), av, dtype=np.int8 if a_s else np.uint8)
                w = np.full((9, 20, 3, 3), wv, dtype=np.int8 if w_s else np.uint8)
                for tight in (0, 1):
                    plan = dnn_plan(bits, bits, a_s, w_s, 3, 0, True, tight=tight)
                    assert np.array_equal(run_conv2d(plan, x, w, 1, 1), direct.conv2d(x, w, 1, 1)), (bits, av, wv, plan)


@pytest.mark.parametrize("shape", [(1, 4, 6, 7, 8, 3, 3, 1, 1), (2, 16, 9, 9, 9, 3, 3, 1, 0), (1, 8, 8, 10, 12, 3, 3, 2, 1),
                                   (1, 5, 5, 5, 8, 1, 1, 1, 0), (1, 33, 7, 30, 8, 3, 3, 1, 1), (2, 34, 5, 28, 16, 3, 3, 1, 1)])
def test_scalar_register_kernel_bipolar(shape):
    n, c, h, w, co, kh, kw, stride, pad = shape
    x, wt = wl.bipolar_case(n, c, h, w, co, kh, kw, tag="s3")
    ref = direct.conv2d(x, wt, stride, pad)
    for m in (3, 0):
        for tight in (0, 1):
            plan = dnn_plan(1, 1, False, False, kw, m, True, bipolar=True, tight=tight)
            for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
                got = run_conv2d(plan, x, wt, stride, pad, fmt, prepacked=(m == 3))
                assert np.array_equal(got, ref), (shape, m, tight, fmt, plan)


def test_scalar_register_kernel_full_layers():
    x, w = wl.config3()
    ref = direct.conv2d(x, w, 1, 1)
    for m in (5, 0):
        plan = dnn_plan(4, 4, True, True, 3, m, True)
        assert np.array_equal(run_conv2d(plan, x, w, 1, 1, hk.FMT_BITDENSE, prepacked=True), ref)
    x, w = wl.config4()
    ref = direct.conv2d(x, w, 1, 1)
    for tight in (0, 1):
        plan = dnn_plan(1, 1, False, False, 3, 0, True, bipolar=True, tight=tight)
        assert np.array_equal(run_conv2d(plan, x, w, 1, 1, hk.FMT_BITDENSE, prepacked=True), ref)


def test_library_picks_the_kernel_for_a_large_layer():
    # without the override: 256 input channels (768 terms) and more than a thousand
    # (row group, channel tile) pairs select the scalar-register kernel; same result either way
    rng = wl.rng_for("s5")
    x = wl.uniform_values(rng, (8, 256, 28, 28), 4, True)
    w = wl.uniform_values(rng, (256, 256, 3, 3), 4, True)
    ref = direct.conv2d(x, w, 1, 1)
    plan = hk.with_fields(dnn_plan(4, 4, True, True, 3, 0, True), kernel=hk.KERNEL_AUTO)
    assert np.array_equal(run_conv2d(plan, x, w, 1, 1, hk.FMT_INT8, prepacked=True), ref)
    plan = hk.with_fields(plan, kernel=hk.KERNEL_LDS)
    assert np.array_equal(run_conv2d(plan, x, w, 1, 1, hk.FMT_INT8, prepacked=True), ref)


@pytest.mark.parametrize("kernel", ["lds", "sreg"])
def test_stores_with_64bit_addresses(kernel):
    """The layer kernels store through 32-bit buffer offsets when a wave's outputs lie within
    2^31 bytes; the plan flag HIKONV_F_STORES64 forces the path for larger windows (plain stores
    with 64-bit addresses) on shapes small enough to check in full."""
    gpu_util.LAYER_DEFAULTS.update(kernel=hk.KERNEL_LDS if kernel == "lds" else hk.KERNEL_SREG, flags=hk.F_STORES64)
    for bits, a_s, w_s in ((4, True, True), (1, False, False), (8, False, True)):
        for shape in SHAPES:
            x, w = _case(bits, a_s, w_s, shape, "s9")
            stride, pad, kw = shape[7], shape[8], shape[6]
            ref = direct.conv2d(x, w, stride, pad)
            plan = dnn_plan(bits, bits, a_s, w_s, kw, 0)
            assert plan.flags == hk.F_STORES64
            assert np.array_equal(run_conv2d(plan, x, w, stride, pad, hk.FMT_INT8), ref), (bits, shape, kernel)
