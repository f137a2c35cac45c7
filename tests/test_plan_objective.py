"""CPU checks of the planner's second objective (modelled VALU issue slots per output on
gfx950 instead of Algorithm 1's operations per multiply), of the container-aligned plans it
can return, and of the constraint that keeps layer plans within what the layer kernels hold.

The container-aligned packing itself (Theorem 1 with K = 1, elements of a word J apart) is
pinned against numpy in test_packed_model_pins.py; here the planner's description of it is
checked against the big-integer model and against exhaustive corner inputs."""
import itertools

import numpy as np
import pytest

import paper_2208_00763_amd as hk
from oracle import plan_model as pl


def conv1d_request(bits, signed, taps, objective, out_bits=0, bits_w=None, w_signed=None, **kw):
    return hk.hikonv_plan_ex(bits_a=bits, bits_w=bits_w or bits, a_signed=int(signed),
                             w_signed=int(signed if w_signed is None else w_signed), L_A=32, L_B=32, L_acc=64,
                             mode=hk.MODE_CONV1D, taps=taps, objective=objective, out_bits=out_bits, **kw)


def test_paper_objective_is_unchanged_by_the_new_fields():
    for b, taps in itertools.product(range(1, 9), (1, 3, 5, 7)):
        got = conv1d_request(b, False, taps, hk.OBJ_PAPER_OPS)
        ref = pl.paper_search_taps(b, b, 32, 32, taps, pl.CONV1D)
        assert (got.N, got.K, got.S, got.G_b, got.chunks) == (ref["N"], ref["K"], ref["S"], ref["G_b"], ref["chunks"])
        assert got.paper_exact == 1 and got.stride_elems == 1
        # the output form is not part of Algorithm 1: out_bits changes nothing under its objective
        same = conv1d_request(b, False, taps, hk.OBJ_PAPER_OPS, out_bits=b)
        assert (same.N, same.K, same.S, same.stride_elems) == (got.N, got.K, got.S, 1)


@pytest.mark.parametrize("bits,signed,expect", [
    (4, False, (2, 1, 16, 4)), (2, False, (2, 1, 16, 8)), (1, False, (8, 1, 4, 4)), (4, True, (2, 1, 16, 4)),
    (3, True, (2, 1, 16, 4)), (1, True, (2, 1, 16, 16)),
])
def test_cost_objective_returns_container_aligned_slices_for_requantised_output(bits, signed, expect):
    plan = conv1d_request(bits, signed, 3, hk.OBJ_MEASURED_COST, out_bits=bits)
    assert (plan.N, plan.K, plan.S, plan.stride_elems) == expect
    assert plan.chunks == 3 and plan.paper_exact == 0
    assert plan.stride_elems * {1: 1, 2: 2, 3: 4, 4: 4}[bits] == plan.S        # J = S / c
    assert hk.hikonv_plan_check(plan) == hk.OK
    assert hk.hikonv_plan_cost(plan) == plan.cost_milli > 0
    paper = conv1d_request(bits, signed, 3, hk.OBJ_PAPER_OPS, out_bits=bits)
    assert hk.hikonv_plan_cost(paper) > plan.cost_milli


def test_cost_objective_keeps_the_plan_slices_where_aligned_slices_are_not_exact():
    # int32 outputs: no container-aligned slices, Algorithm 1's plan (the path is memory-bound)
    plan = conv1d_request(4, False, 3, hk.OBJ_MEASURED_COST, out_bits=0)
    assert plan.stride_elems == 1 and plan.K > 1
    # 3 taps of 8-bit unsigned products reach 195075 > 2^16 - 1; other containers in and out: no aligned
    # slices either, and with requantised outputs no packed plan is then cheaper than one product per
    # multiply (measured, 4096 x 65536, 3 taps, 8 bit: Algorithm 1's plan 0.31 ms, the one-product kernel
    # 0.16 ms): the objective answers with Theorem 1's smallest case, N = K = 1
    assert conv1d_request(4, False, 3, hk.OBJ_MEASURED_COST, out_bits=8).stride_elems == 1
    for kw in (dict(bits=8, signed=False, out_bits=8), dict(bits=8, signed=True, out_bits=8)):
        plan = conv1d_request(kw["bits"], kw["signed"], 3, hk.OBJ_MEASURED_COST, out_bits=kw["out_bits"])
        assert (plan.N, plan.K, plan.stride_elems, plan.chunks) == (1, 1, 1, 3)
        assert hk.hikonv_plan_check(plan) == hk.OK
        paper = conv1d_request(kw["bits"], kw["signed"], 3, hk.OBJ_PAPER_OPS, out_bits=kw["out_bits"])
        assert paper.K > 1 and hk.hikonv_plan_cost(paper) > plan.cost_milli
    # 7-bit signed, 5 taps: 5 * 64 * 64 = 20480 < 2^15 fits and the window of 4 + 4 bytes is 64 bits;
    # 6 taps: the window would be 72 bits
    assert conv1d_request(7, True, 5, hk.OBJ_MEASURED_COST, out_bits=7).stride_elems == 2
    assert conv1d_request(7, True, 6, hk.OBJ_MEASURED_COST, out_bits=7).stride_elems == 1
    # 6-bit unsigned, 5 taps: 5 * 63 * 63 = 19845 fits 16 bits; 8-bit unsigned x 2-bit: 3 * 255 * 3 fits
    assert conv1d_request(6, False, 5, hk.OBJ_MEASURED_COST, out_bits=6).stride_elems == 2
    assert conv1d_request(8, False, 3, hk.OBJ_MEASURED_COST, out_bits=8, bits_w=2).stride_elems == 2
    # 4-bit, 8 taps: beyond the kernel's 7
    assert conv1d_request(4, False, 8, hk.OBJ_MEASURED_COST, out_bits=4).stride_elems == 1


def test_aligned_plan_check_is_the_exact_bound():
    """hikonv_plan_check on container-aligned plans: accepted exactly when taps * max|a| * max|w|
    fits the slice (2^16 - 1 unsigned; +-(2^15 - 1) signed), all operand widths and signs."""
    for p, q, a_s, w_s, taps in itertools.product(range(1, 9), range(1, 9), (0, 1), (0, 1), (1, 3, 7)):
        lo_a, hi_a = (-(1 << (p - 1)), (1 << (p - 1)) - 1) if a_s else (0, (1 << p) - 1)
        lo_w, hi_w = (-(1 << (q - 1)), (1 << (q - 1)) - 1) if w_s else (0, (1 << q) - 1)
        prods = [a * w for a in (lo_a, hi_a) for w in (lo_w, hi_w)]
        lo, hi = taps * min(prods), taps * max(prods)
        c = {1: 1, 2: 2, 3: 4, 4: 4}.get(p, 8)
        if a_s or w_s:
            fits = -(2 ** 15 - 1) <= lo and hi <= 2 ** 15 - 1 and p <= 7
        else:
            fits = hi <= 2 ** 16 - 1
        fits = fits and (32 // c + taps - 1) * c <= 64
        plan = hk.Plan(bits_a=p, bits_w=q, a_signed=a_s, w_signed=w_s, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_CONV1D,
                       taps=taps, out_bits=p, N=2, K=1, S=16, chunks=taps, stride_elems=16 // c)
        assert (hk.hikonv_plan_check(plan) == hk.OK) == fits, (p, q, a_s, w_s, taps)
    # nibble slices: one-bit unsigned operands, at most 7 taps
    nib = dict(bits_a=1, bits_w=1, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_CONV1D, out_bits=1, N=8, K=1, S=4,
               stride_elems=4)
    assert hk.hikonv_plan_check(hk.Plan(taps=7, chunks=7, **nib)) == hk.OK
    assert hk.hikonv_plan_check(hk.Plan(taps=8, chunks=8, **nib)) != hk.OK
    assert hk.hikonv_plan_check(hk.Plan(taps=3, chunks=3, **dict(nib, a_signed=1))) != hk.OK
    # a description that is not the one form per slice width is refused
    bad = hk.Plan(bits_a=4, bits_w=4, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_CONV1D, taps=3, out_bits=4, N=2, K=1, S=16,
                  chunks=3, stride_elems=2)
    assert hk.hikonv_plan_check(bad) == hk.EINVAL


def test_aligned_plans_are_exact_in_the_big_integer_model_on_corner_inputs():
    """The plan's (N, K = 1, S, stride J): word rho of a window holds elements rho and rho + J (, ...);
    Y_rho = sum_k A_(rho + taps-1-k) g[k]; its slices are outputs rho + n*J.  All-extreme inputs."""
    for bits, signed, taps in ((4, False, 3), (4, True, 3), (2, False, 7), (1, False, 7), (7, True, 5), (6, False, 5)):
        plan = conv1d_request(bits, signed, taps, hk.OBJ_MEASURED_COST, out_bits=bits)
        assert plan.stride_elems > 1
        n_s, s_bits, j = plan.N, plan.S, plan.stride_elems
        lo, hi = (-(1 << (bits - 1)), (1 << (bits - 1)) - 1) if signed else (0, (1 << bits) - 1)
        for fv, gv in itertools.product((lo, hi), repeat=2):
            f = [fv] * (n_s * j + taps - 1)           # the window of one output dword's worth of slices
            g = [gv] * taps
            ref = np.convolve(np.array(f, dtype=np.int64), np.array(g, dtype=np.int64), mode="valid")
            for rho in range(j):
                y = 0
                for k in range(taps):
                    tau = rho + taps - 1 - k
                    a_word = sum(f[tau + n * j] << (s_bits * n) for n in range(n_s))      # shift + mask of the window
                    y += a_word * g[k]
                for n in range(n_s):                   # split: sign-extended field plus the bit below it
                    field = (y >> (s_bits * n)) & ((1 << s_bits) - 1)
                    if signed:
                        field = field - (1 << s_bits) if field >> (s_bits - 1) else field
                        if n > 0:
                            field += (y >> (s_bits * n - 1)) & 1
                    assert field == ref[rho + n * j], (bits, signed, taps, fv, gv, rho, n)


# Measured on one MI355X, 4096 rows x 65536, 3 taps, valid, requantised bit-dense output at the
# input's width (milliseconds per launch; bench.py, conv1d_requant_bitdense_out):
# (bits, signed) -> (container-aligned slices, the paper's plan)
MEASURED_REQUANT_MS = {(4, False): (0.050, 0.163), (2, False): (0.040, 0.136), (1, False): (0.022, 0.132),
                       (4, True): (0.057, 0.169)}


def test_cost_ranking_reproduces_the_measured_ranking():
    """For every benchmarked requantising case the model orders the two plans as the clock does,
    and its cost ratio is within a factor 1.6 of the measured time ratio (both kernels are
    ALU-bound there, so slots per output is what the time follows)."""
    for (bits, signed), (ms_aligned, ms_paper) in MEASURED_REQUANT_MS.items():
        aligned = conv1d_request(bits, signed, 3, hk.OBJ_MEASURED_COST, out_bits=bits)
        paper = conv1d_request(bits, signed, 3, hk.OBJ_PAPER_OPS, out_bits=bits)
        assert aligned.stride_elems > 1 and paper.stride_elems == 1
        ca, cp = hk.hikonv_plan_cost(aligned), hk.hikonv_plan_cost(paper)
        assert (ca < cp) == (ms_aligned < ms_paper)
        assert 1 / 1.6 < (cp / ca) / (ms_paper / ms_aligned) < 1.6, (bits, signed, cp / ca, ms_paper / ms_aligned)
    # across the widths the aligned plans also rank as measured: 1 bit < 2 bit < 4 bit < 4 bit signed
    order = [conv1d_request(b, s, 3, hk.OBJ_MEASURED_COST, out_bits=b).cost_milli
             for b, s in ((1, False), (2, False), (4, False), (4, True))]
    assert order == sorted(order)


def test_int32_output_plans_sit_under_the_memory_floor():
    """With int32 outputs every candidate of the sweep needs fewer issue slots than pass during
    the HBM time of its 4 + c/8 bytes per output (4.9 slots per byte at the published peaks), so
    the cost objective ties them at the floor, where Algorithm 1's own order decides: the sweep's
    int32 plans are the same under both objectives."""
    for b, signed in itertools.product(range(1, 9), (False, True)):
        cost = conv1d_request(b, signed, 3, hk.OBJ_MEASURED_COST)
        paper = conv1d_request(b, signed, 3, hk.OBJ_PAPER_OPS)
        assert (cost.N, cost.K, cost.S, cost.stride_elems) == (paper.N, paper.K, paper.S, 1)
        c = {1: 1, 2: 2, 3: 4, 4: 4}.get(b, 8)
        floor_milli = (4 + c / 8) * 256 * 64 * 2.4e9 / 8e12 * 1000
        if cost.chunks == 1:
            assert cost.cost_milli < floor_milli


def test_max_n_bounds_layer_plans():
    """The layer kernels hold at most LAYER_MAX_N slices per lane.  Unbounded, the one-bit
    DNN search returns more; with max_N the planner stays inside, and the bounded plan is the
    best of the plans with N <= max_N."""
    free = hk.hikonv_plan_ex(bits_a=1, bits_w=1, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_DNN, M=1, taps=3)
    assert free.N > hk.LAYER_MAX_N
    bounded = hk.hikonv_plan_ex(bits_a=1, bits_w=1, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_DNN, M=1, taps=3,
                                max_N=hk.LAYER_MAX_N)
    assert bounded.N == hk.LAYER_MAX_N and bounded.paper_exact == 0
    assert hk.hikonv_plan_check(bounded) == hk.OK
    # the layer entry points refuse the unbounded plan on the host, before anything is launched
    # (no device pointer is touched: the arguments here are null), and size a workspace for the bounded one
    import ctypes as C
    assert hk.hikonv_conv2d_workspace_bytes(free, 1, 4, 8, 8, 8, 3, 3, 1, 1, False) == 0
    assert hk.hikonv_conv2d_workspace_bytes(bounded, 1, 4, 8, 8, 8, 3, 3, 1, 1, False) > 0
    rc = hk.lib.hikonv_conv2d(C.byref(free), None, hk.FMT_INT8, 1, 4, 8, 8, None, 8, 3, 3, 1, 1, None, 0, None, None)
    assert rc == hk.EUNSUPPORTED
    rc = hk.lib.hikonv_conv2d_noalloc(C.byref(free), None, hk.FMT_INT8, 1, 4, 8, 8, None, 8, 3, 3, 1, 1, None, None)
    assert rc == hk.EUNSUPPORTED
    for b, m in itertools.product(range(1, 9), (1, 4, 16, 0)):
        p = hk.hikonv_plan_ex(bits_a=b, bits_w=b, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_DNN, M=m, taps=3, max_N=5)
        assert 1 <= p.N <= 5
    with pytest.raises(hk.HikonvError):
        hk.hikonv_plan_ex(bits_a=1, bits_w=1, L_A=32, L_B=32, mode=hk.MODE_DNN, M=1, taps=3, max_N=65)


def test_request_fields_are_validated_and_copied_through():
    p = hk.hikonv_plan_ex(bits_a=4, bits_w=4, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_DNN, M=0, taps=3,
                          kernel=hk.KERNEL_SREG, flags=hk.F_STORES64, max_N=8)
    assert (p.kernel, p.flags, p.max_N) == (hk.KERNEL_SREG, hk.F_STORES64, 8)
    for bad in (dict(objective=2), dict(objective=-1), dict(out_bits=9), dict(out_bits=-1), dict(kernel=5), dict(kernel=-1),
                dict(flags=2), dict(max_N=-1)):
        with pytest.raises(hk.HikonvError) as e:
            hk.hikonv_plan_ex(bits_a=4, bits_w=4, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_CONV1D, taps=3, **bad)
        assert e.value.code == hk.EINVAL
    assert hk.hikonv_plan_cost(hk.hikonv_plan(4, 4, 0, 32)) == hk.EUNSUPPORTED      # single-multiplier plan: no kernel to price


# Layer plans (mode DNN).  Measured on one MI355X, layer 8x256x28x28 -> 256, 3x3, int4 signed, packed
# input: Algorithm 1's plan (N=3, K=3, S=13, M=10) 54 us, the exact-interval plan (M=21) 40 us.
MEASURED_INT4_LAYER_US = (40.0, 54.0)


def layer_request(objective, tight=0, **kw):
    base = dict(L_A=32, L_B=32, L_acc=64, mode=hk.MODE_DNN, M=0, taps=3, objective=objective, tight=tight,
                max_N=hk.LAYER_MAX_N)
    base.update(kw)
    return hk.hikonv_plan_ex(**base)


def test_layer_cost_objective_finds_the_exact_interval_plans():
    """In DNN mode the cost objective prices splits and extra B words; what it returns is the plan
    that `tight` asks for by hand (more products per split, or more slices per word), never a costlier
    one than Algorithm 1's."""
    cases = (dict(bits_a=4, bits_w=4, a_signed=1, w_signed=1), dict(bits_a=4, bits_w=4, w_signed=1),
             dict(bits_a=8, bits_w=8, a_signed=1, w_signed=1), dict(bits_a=2, bits_w=2), dict(bits_a=1, bits_w=1),
             dict(bits_a=1, bits_w=1, bipolar=1), dict(bits_a=3, bits_w=5, w_signed=1))
    for kw in cases:
        paper = layer_request(hk.OBJ_PAPER_OPS, **kw)
        tight = layer_request(hk.OBJ_PAPER_OPS, tight=1, **kw)
        cost = layer_request(hk.OBJ_MEASURED_COST, **kw)
        assert (cost.N, cost.K, cost.S, cost.M, cost.chunks) == (tight.N, tight.K, tight.S, tight.M, tight.chunks), kw
        assert hk.hikonv_plan_check(cost) == hk.OK
        assert cost.cost_milli == hk.hikonv_plan_cost(cost) <= hk.hikonv_plan_cost(paper), kw
        if (cost.N, cost.S, cost.M) != (paper.N, paper.S, paper.M):
            assert cost.paper_exact == 0


def test_layer_cost_ranking_reproduces_the_measured_ranking():
    kw = dict(bits_a=4, bits_w=4, a_signed=1, w_signed=1)
    paper, cost = layer_request(hk.OBJ_PAPER_OPS, **kw), layer_request(hk.OBJ_MEASURED_COST, **kw)
    assert (paper.M, cost.M) == (10, 21)
    model = hk.hikonv_plan_cost(paper) / hk.hikonv_plan_cost(cost)
    clock = MEASURED_INT4_LAYER_US[1] / MEASURED_INT4_LAYER_US[0]
    assert model > 1.0 and clock > 1.0
    assert 1 / 1.3 < model / clock < 1.3
