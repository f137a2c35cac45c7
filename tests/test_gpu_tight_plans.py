"""GPU parity for plans with the smallest provably exact slice (tight = 1): more values per
word or more products per split than Eq. (slice1) allows, still bit-exact - on random data and
on the all-minimum / all-maximum inputs that fill every segment to its bound."""
import itertools

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import direct

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_00763_amd as hk
    from gpu_util import run_conv1d, run_conv2d, oracle_conv1d, conv1d_plan, dnn_plan

SIGNS = [(False, False), (True, True), (False, True), (True, False)]


@pytest.mark.parametrize("bits", range(1, 9))
@pytest.mark.parametrize("signs", SIGNS)
def test_conv1d_tight_plans(bits, signs):
    a_s, w_s = signs
    for taps in (1, 3, 5, 7):
        plan = conv1d_plan(bits, a_s, w_s, taps, tight=1)
        loose = conv1d_plan(bits, a_s, w_s, taps)
        assert plan.N * loose.chunks >= loose.N * plan.chunks
        rng = wl.rng_for("tight1", bits, signs, taps)
        for rows, length in ((3, 1000), (2, 20011)):
            x = wl.uniform_values(rng, (rows, length), bits, a_s)
            g = wl.uniform_values(rng, (taps,), bits, w_s)
            for mode in (hk.OUT_FULL, hk.OUT_VALID):
                ref = oracle_conv1d(x, g, mode)
                for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
                    got = run_conv1d(x, g, bits, a_s, w_s, mode, fmt, plan=plan)
                    assert np.array_equal(got, ref), (bits, signs, taps, length, mode, fmt, plan)
        for av, gv in itertools.product(wl.value_range(bits, a_s), wl.value_range(bits, w_s)):
            x = np.full((2, 3001), av, dtype=np.int8 if a_s else np.uint8)
            g = np.full((taps,), gv, dtype=np.int8 if w_s else np.uint8)
            got = run_conv1d(x, g, bits, a_s, w_s, hk.OUT_FULL, hk.FMT_BITDENSE, plan=plan)
            assert np.array_equal(got, oracle_conv1d(x, g, hk.OUT_FULL)), (bits, signs, taps, av, gv, plan)


def test_conv1d_tight_signed_4bit_plan_and_full_size_rows():
    plan = conv1d_plan(4, True, True, 3, tight=1)
    assert (plan.N, plan.K, plan.S, plan.paper_exact) == (4, 3, 9, 0)
    x, g = wl.conv1d_case(4, True, 3, 4096, 65536)
    sample = np.array([0, 1, 2048, 4095] + list(wl.rng_for("tight_rows").integers(0, 4096, 12)))
    from gpu_util import compact, dev
    x_d, g_d = compact(x, 4), dev(g)
    out_len = 65536 - 2
    y = torch.empty(4096 * out_len, dtype=torch.int32, device="cuda")
    hk.hikonv_conv1d(plan, x_d, hk.FMT_BITDENSE, 4096, 65536, g_d, 3, hk.OUT_VALID, y)
    torch.cuda.synchronize()
    got = y.view(4096, out_len)[torch.from_numpy(sample).cuda()].cpu().numpy()
    assert np.array_equal(got, direct.conv1d(x[sample], g, direct.VALID))


@pytest.mark.parametrize("how", ["tight", "cost_objective"])
@pytest.mark.parametrize("wide", [True, False])
def test_conv2d_tight_plans_random_and_extreme(wide, how):
    # the exact-interval slices, asked for directly and as the planner's cost objective finds them
    request = dict(tight=1) if how == "tight" else dict(objective=hk.OBJ_MEASURED_COST)
    for bits, a_s, w_s in ((4, True, True), (4, False, True), (4, False, False), (2, True, True), (3, False, True),
                           (8, True, True)):
        try:
            plan = dnn_plan(bits, bits, a_s, w_s, 3, 0, wide, **request)
        except hk.HikonvError as e:
            assert e.code == hk.ENOPLAN    # no plan exists for this request; nothing is skipped silently
            continue
        c = min(max(plan.M // 3 + 2, 8), 160)      # at least one full split group of (channel, row) terms
        x, w = wl.conv2d_case(bits, a_s, w_s, 1, c, 9, 21, 10, 3, 3, tag="tight2")
        assert np.array_equal(run_conv2d(plan, x, w, 1, 1), direct.conv2d(x, w, 1, 1)), (bits, a_s, w_s, plan)
        for av, wv in itertools.product(wl.value_range(bits, a_s), wl.value_range(bits, w_s)):
            x = np.full((1, c, 6, 9), av, dtype=np.int8 if a_s else np.uint8)
            w = np.full((3, c, 3, 3), wv, dtype=np.int8 if w_s else np.uint8)
            assert np.array_equal(run_conv2d(plan, x, w, 1, 1), direct.conv2d(x, w, 1, 1)), (bits, av, wv, plan)


def test_conv2d_tight_config3_and_config4_full():
    x, w = wl.config3()
    plan = dnn_plan(4, 4, True, True, 3, 0, True, tight=1)
    assert plan.M > dnn_plan(4, 4, True, True, 3, 0, True).M and plan.paper_exact == 0
    assert np.array_equal(run_conv2d(plan, x, w, 1, 1, hk.FMT_BITDENSE, prepacked=True), direct.conv2d(x, w, 1, 1))
    x, w = wl.config4()
    ref = direct.conv2d(x, w, 1, 1)
    for wide in (True, False):
        plan = dnn_plan(1, 1, False, False, 3, 0, wide, bipolar=True, tight=1)
        assert np.array_equal(run_conv2d(plan, x, w, 1, 1, hk.FMT_BITDENSE, prepacked=True), ref), plan
    # all +1 / all -1 activations and weights: every segment at its bound
    for av, wv in itertools.product((-1, 1), (-1, 1)):
        xe = np.full((1, 256, 6, 14), av, dtype=np.int8)
        we = np.full((8, 256, 3, 3), wv, dtype=np.int8)
        plan = dnn_plan(1, 1, False, False, 3, 0, True, bipolar=True, tight=1)
        assert np.array_equal(run_conv2d(plan, xe, we, 1, 1), direct.conv2d(xe, we, 1, 1)), (av, wv, plan)
