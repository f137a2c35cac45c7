"""GPU parity with different widths for activations and weights (p != q in Eq. slice1; the
paper evaluates p = q only), including its 1-bit special cases S = q + G_b / p + G_b."""
import itertools

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import direct

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_00763_amd as hk
    from gpu_util import run_conv1d, run_conv2d, oracle_conv1d, conv1d_plan

WIDTHS = [(1, 4), (4, 1), (2, 8), (8, 2), (4, 8), (8, 4), (3, 5), (1, 8), (6, 2)]
SIGNS = [(False, False), (True, True), (False, True), (True, False)]


@pytest.mark.parametrize("widths", WIDTHS)
@pytest.mark.parametrize("tight", [0, 1])
def test_conv1d_mixed_widths(widths, tight):
    p, q = widths
    for (a_s, w_s), taps in itertools.product(SIGNS, (1, 3, 5)):
        plan = conv1d_plan(p, a_s, w_s, taps, tight=tight, bits_w=q)
        assert (plan.bits_a, plan.bits_w) == (p, q)
        rng = wl.rng_for("mixed1", p, q, a_s, w_s, taps)
        x = wl.uniform_values(rng, (3, 4099), p, a_s)
        g = wl.uniform_values(rng, (taps,), q, w_s)
        for mode in (hk.OUT_FULL, hk.OUT_VALID):
            ref = oracle_conv1d(x, g, mode)
            for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
                got = run_conv1d(x, g, p, a_s, w_s, mode, fmt, plan=plan)
                assert np.array_equal(got, ref), (widths, a_s, w_s, taps, mode, fmt, plan)
        for av, gv in itertools.product(wl.value_range(p, a_s), wl.value_range(q, w_s)):
            x = np.full((1, 700), av, dtype=np.int8 if a_s else np.uint8)
            g = np.full((taps,), gv, dtype=np.int8 if w_s else np.uint8)
            got = run_conv1d(x, g, p, a_s, w_s, hk.OUT_FULL, hk.FMT_BITDENSE, plan=plan)
            assert np.array_equal(got, oracle_conv1d(x, g, hk.OUT_FULL)), (widths, a_s, w_s, taps, av, gv, plan)


@pytest.mark.parametrize("widths", WIDTHS)
@pytest.mark.parametrize("wide", [True, False])
def test_conv2d_mixed_widths(widths, wide):
    p, q = widths
    width = 32 if wide else 24
    for (a_s, w_s), tight in itertools.product(SIGNS, (0, 1)):
        try:
            plan = hk.hikonv_plan_ex(bits_a=p, bits_w=q, a_signed=int(a_s), w_signed=int(w_s), L_A=width, L_B=width,
                                     L_acc=64 if wide else 32, mode=hk.MODE_DNN, M=0, taps=3, tight=tight,
                                     max_N=hk.LAYER_MAX_N)
        except hk.HikonvError as e:
            assert e.code == hk.ENOPLAN
            continue
        rng = wl.rng_for("mixed2", p, q, a_s, w_s, wide, tight)
        c = min(max(plan.M // 3 + 2, 6), 120)
        x = wl.uniform_values(rng, (1, c, 7, 23), p, a_s)
        w = wl.uniform_values(rng, (5, c, 3, 3), q, w_s)
        for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
            assert np.array_equal(run_conv2d(plan, x, w, 1, 1, fmt), direct.conv2d(x, w, 1, 1)), (widths, a_s, w_s, plan)
        for av, wv in itertools.product(wl.value_range(p, a_s), wl.value_range(q, w_s)):
            x = np.full((1, c, 5, 9), av, dtype=np.int8 if a_s else np.uint8)
            w = np.full((2, c, 3, 3), wv, dtype=np.int8 if w_s else np.uint8)
            assert np.array_equal(run_conv2d(plan, x, w, 1, 1), direct.conv2d(x, w, 1, 1)), (widths, av, wv, plan)
