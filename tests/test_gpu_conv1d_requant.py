"""GPU parity: 1-D convolution with in-kernel requantisation and bit-dense output through the
C ABI vs the oracle chain direct convolution -> ReLU/shift/clamp -> bit-dense packing,
byte for byte (padding bits of every row included)."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import direct

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_00763_amd as hk
    from gpu_util import compact, dev, Guarded

SIGNS = [(False, False), (True, True), (False, True), (True, False)]
GUARD = 0xA5


OBJECTIVE = {"value": 0}


@pytest.fixture(autouse=True, params=["measured_cost", "paper_ops"])
def objective(request):
    """Every case runs twice: with the plan of the measured-cost objective (container-aligned
    slices where input and output containers are equal and the sums fit) and with Algorithm 1's."""
    OBJECTIVE["value"] = hk.OBJ_MEASURED_COST if request.param == "measured_cost" else hk.OBJ_PAPER_OPS
    yield request.param
    OBJECTIVE["value"] = 0


def requant_plan(bits, a_s, w_s, taps, out_bits, bits_w=None, fmt=None):
    """The plan of the objective under test.  The planner prices bit-dense inputs; for inputs
    stored one value per byte the containers differ from what it assumed, so a container-aligned
    plan does not describe that call (the entry point refuses it) and Algorithm 1's plan is taken."""
    kw = dict(bits_a=bits, bits_w=bits_w or bits, a_signed=int(a_s), w_signed=int(w_s), L_A=32, L_B=32, L_acc=64,
              mode=hk.MODE_CONV1D, taps=taps, out_bits=out_bits)
    plan = hk.hikonv_plan_ex(objective=OBJECTIVE["value"], **kw)
    if fmt == hk.FMT_INT8 and plan.stride_elems > 1 and bits < 5:
        plan = hk.hikonv_plan_ex(objective=hk.OBJ_PAPER_OPS, **kw)
    return plan


def oracle_requant(x, g, mode, shift, qmax, out_bits):
    y = direct.conv1d(x, g, direct.FULL if mode == hk.OUT_FULL else direct.VALID)
    if y.shape[1] == 0:
        return np.zeros((x.shape[0], 0), dtype=np.uint8)
    return direct.bitdense_pack(direct.relu_requant(y, shift, qmax), out_bits)


def run_requant(x, g, bits, a_s, w_s, mode, fmt, shift, qmax, out_bits, packed=True):
    rows, length = x.shape
    taps = g.shape[0]
    out_len = length + taps - 1 if mode == hk.OUT_FULL else max(length - taps + 1, 0)
    row_bytes = hk.hikonv_bitdense_row_bytes(out_len, out_bits) if out_len else 0
    out = Guarded(rows * row_bytes, torch.uint8, GUARD)
    q = out.view
    x_d = compact(x, bits) if fmt == hk.FMT_BITDENSE else dev(x)
    g_d = dev(g)
    if packed:
        plan = requant_plan(bits, a_s, w_s, taps, out_bits, fmt=fmt)
        hk.hikonv_conv1d_requant(plan, x_d, fmt, rows, length, g_d, taps, mode, shift, qmax, out_bits, q)
    else:
        hk.hikonv_conv1d_requant_unpacked(bits, bits, hk.signedness(a_s, w_s), x_d, fmt, rows, length, g_d, taps,
                                          mode, shift, qmax, out_bits, q)
    return out.result().reshape(rows, row_bytes)


def values(tag, bits, a_s, w_s, taps, rows, length):
    rng = wl.rng_for(tag, bits, a_s, w_s, taps, rows, length)
    return wl.uniform_values(rng, (rows, length), bits, a_s), wl.uniform_values(rng, (taps,), bits, w_s)


def pick_shift(bits, taps, out_bits):
    """A shift that leaves some outputs clamped and some not."""
    top = taps * ((1 << bits) - 1) ** 2
    return max(0, int(top).bit_length() - out_bits - 1)


@pytest.mark.parametrize("bits", range(1, 9))
@pytest.mark.parametrize("signs", SIGNS)
def test_requant_small_shapes(bits, signs):
    a_s, w_s = signs
    for taps in (1, 2, 3, 5, 7):
        for length in (1, 2, 6, 97, 1000):
            x, g = values("rq1", bits, a_s, w_s, taps, 3, length)
            for mode in (hk.OUT_FULL, hk.OUT_VALID):
                out_bits = (1, 2, 4, 3, 7)[(taps + length + mode) % 5]
                qmax = (1 << out_bits) - 1
                shift = pick_shift(bits, taps, out_bits)
                ref = oracle_requant(x, g, mode, shift, qmax, out_bits)
                for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
                    for packed in (True, False):
                        got = run_requant(x, g, bits, a_s, w_s, mode, fmt, shift, qmax, out_bits, packed)
                        assert got.shape == ref.shape
                        assert np.array_equal(got, ref), (bits, signs, taps, length, mode, fmt, packed, out_bits)


@pytest.mark.parametrize("bits,signs,taps,out_bits", [
    (1, (False, False), 3, 1), (1, (True, True), 7, 2), (2, (True, True), 3, 2), (4, (False, False), 3, 4),
    (4, (True, True), 5, 4), (3, (False, True), 3, 1), (6, (True, True), 3, 4), (8, (False, False), 7, 7),
    (8, (True, True), 3, 4), (4, (False, False), 9, 2), (2, (False, False), 13, 4)])
def test_requant_several_runs_and_ragged_tail(bits, signs, taps, out_bits):
    a_s, w_s = signs
    for rows, length in ((5, 20011), (2, 65536), (7, 4099), (3, 1511)):
        x, g = values("rq2", bits, a_s, w_s, taps, rows, length)
        for mode in (hk.OUT_FULL, hk.OUT_VALID):
            for shift in (0, pick_shift(bits, taps, out_bits)):
                qmax = (1 << out_bits) - 1
                ref = oracle_requant(x, g, mode, shift, qmax, out_bits)
                for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
                    assert np.array_equal(run_requant(x, g, bits, a_s, w_s, mode, fmt, shift, qmax, out_bits), ref)
                got = run_requant(x, g, bits, a_s, w_s, mode, hk.FMT_BITDENSE, shift, qmax, out_bits, packed=False)
                assert np.array_equal(got, ref)


@pytest.mark.parametrize("bits,signed", [(1, False), (2, True), (4, False), (4, True), (8, True)])
def test_requant_extreme_values_and_partial_clamp(bits, signed):
    lo, hi = wl.value_range(bits, signed)
    taps, length = 3, 3000
    for xv, gv in ((hi, hi), (lo, lo), (lo, hi), (hi, lo)):
        x = np.full((2, length), xv, dtype=np.int8 if signed else np.uint8)
        g = np.full((taps,), gv, dtype=np.int8 if signed else np.uint8)
        for qmax, out_bits, shift in ((5, 3, 0), (1, 1, 2), (100, 8, 1), (0, 2, 0)):
            ref = oracle_requant(x, g, hk.OUT_FULL, shift, qmax, out_bits)
            for packed in (True, False):
                got = run_requant(x, g, bits, signed, signed, hk.OUT_FULL, hk.FMT_BITDENSE, shift, qmax, out_bits,
                                  packed)
                assert np.array_equal(got, ref), (bits, signed, xv, gv, qmax, out_bits, shift, packed)


@pytest.mark.parametrize("signed", [False, True])
def test_requant_shift_at_and_beyond_the_slice_width(signed):
    """Shifts around S (10 for 4-bit, 3 taps; 16 for the container-aligned slices) up to 31: everything
    ends at 0 or at the last value bit."""
    x, g = values("rq5", 4, signed, signed, 3, 4, 5000)
    for shift in (6, 7, 8, 9, 10, 11, 14, 15, 16, 17, 31):
        ref = oracle_requant(x, g, hk.OUT_VALID, shift, 15, 4)
        for packed in (True, False):
            got = run_requant(x, g, 4, signed, signed, hk.OUT_VALID, hk.FMT_BITDENSE, shift, 15, 4, packed)
            assert np.array_equal(got, ref), (signed, shift, packed)


@pytest.mark.parametrize("bits,signed", [(4, False), (1, False), (2, False), (4, True)])
def test_requant_full_size_all_rows(bits, signed):
    """The benchmark's four cases in its launch configuration: 4096 x 65536, 3 taps, valid,
    bit-dense in and out at the same width, shift and clamp as in bench.py.  Every byte of every
    output row (padding bits included) is compared with the oracle chain, on the device, for the
    packed kernel of the objective under test and for the unpacked baseline."""
    taps, rows, length = 3, 4096, 65536
    x, g = wl.conv1d_case(bits, signed, taps, rows, length)
    shift, qmax, out_bits = max(0, 2 * bits - 3), (1 << bits) - 1, bits
    x_d, g_d = compact(x, bits), dev(g)
    out_len = length - taps + 1
    row_bytes = hk.hikonv_bitdense_row_bytes(out_len, out_bits)
    ref_d = torch.from_numpy(oracle_requant(x, g, hk.OUT_VALID, shift, qmax, out_bits)).cuda().view(-1)
    plan = requant_plan(bits, signed, signed, taps, out_bits)
    assert (plan.stride_elems > 1) == (OBJECTIVE["value"] == hk.OBJ_MEASURED_COST)
    for packed in (True, False):
        out = Guarded(rows * row_bytes, torch.uint8, GUARD)
        if packed:
            hk.hikonv_conv1d_requant(plan, x_d, hk.FMT_BITDENSE, rows, length, g_d, taps, hk.OUT_VALID, shift, qmax,
                                     out_bits, out.view)
        else:
            hk.hikonv_conv1d_requant_unpacked(bits, bits, hk.signedness(signed, signed), x_d, hk.FMT_BITDENSE, rows,
                                              length, g_d, taps, hk.OUT_VALID, shift, qmax, out_bits, out.view)
        torch.cuda.synchronize()
        out.check()
        if not torch.equal(out.view, ref_d):
            bad = torch.nonzero(out.view != ref_d)[0].item()
            raise AssertionError((bits, signed, packed, "row %d byte %d" % (bad // row_bytes, bad % row_bytes)))
        # a sizeable share of the outputs is neither 0 nor clamped, so the comparison means something
    vals = ref_d[:row_bytes * 8].cpu().numpy()
    assert 0 < np.count_nonzero(vals) < vals.size


def test_requant_full_size_full_mode_sampled_rows():
    """FULL outputs at the benchmark's size (the row ends differ from VALID): sampled whole rows."""
    bits, taps, rows, length = 4, 3, 4096, 65536
    x, g = wl.conv1d_case(bits, False, taps, rows, length)
    shift, qmax, out_bits = 5, 15, 4
    x_d, g_d = compact(x, bits), dev(g)
    out_len = length + taps - 1
    row_bytes = hk.hikonv_bitdense_row_bytes(out_len, out_bits)
    sample = [0, 1, 2047, 4094, 4095] + list(wl.rng_for("rq_rows").integers(0, rows, 24))
    ref = oracle_requant(x[sample], g, hk.OUT_FULL, shift, qmax, out_bits)
    plan = requant_plan(bits, False, False, taps, out_bits)
    out = Guarded(rows * row_bytes, torch.uint8, GUARD)
    hk.hikonv_conv1d_requant(plan, x_d, hk.FMT_BITDENSE, rows, length, g_d, taps, hk.OUT_FULL, shift, qmax, out_bits,
                             out.view)
    torch.cuda.synchronize()
    out.check()
    got = out.view.view(rows, row_bytes)[sample].cpu().numpy()
    assert np.array_equal(got, ref)


def test_requant_empty_and_rejected_arguments():
    x, g = values("rq4", 4, False, False, 3, 2, 64)
    plan = requant_plan(4, False, False, 3, 4, fmt=hk.FMT_INT8)
    q = torch.full((256,), GUARD, dtype=torch.uint8, device="cuda")
    x_d, g_d = dev(x), dev(g)
    # nothing to do: no rows, no elements, VALID shorter than the kernel
    hk.hikonv_conv1d_requant(plan, x_d, hk.FMT_INT8, 0, 64, g_d, 3, hk.OUT_FULL, 0, 15, 4, q)
    hk.hikonv_conv1d_requant(plan, x_d, hk.FMT_INT8, 2, 0, g_d, 3, hk.OUT_FULL, 0, 15, 4, q)
    hk.hikonv_conv1d_requant(plan, x_d, hk.FMT_INT8, 2, 2, g_d, 3, hk.OUT_VALID, 0, 15, 4, q)
    torch.cuda.synchronize()
    assert (q == GUARD).all()
    for shift, qmax, out_bits in ((-1, 15, 4), (32, 15, 4), (0, 16, 4), (0, -1, 4), (0, 1, 0), (0, 1, 9)):
        with pytest.raises(hk.HikonvError) as e:
            hk.hikonv_conv1d_requant(plan, x_d, hk.FMT_INT8, 2, 64, g_d, 3, hk.OUT_FULL, shift, qmax, out_bits, q)
        assert e.value.code == hk.EINVAL
        with pytest.raises(hk.HikonvError) as e:
            hk.hikonv_conv1d_requant_unpacked(4, 4, 0, x_d, hk.FMT_INT8, 2, 64, g_d, 3, hk.OUT_FULL, shift, qmax,
                                              out_bits, q)
        assert e.value.code == hk.EINVAL
    torch.cuda.synchronize()
    assert (q == GUARD).all()


@pytest.mark.parametrize("p_bits,q_bits,signs", [(1, 4, (False, False)), (1, 1, (False, False)), (4, 2, (False, True)),
                                                 (2, 6, (True, True)), (7, 3, (False, False)), (3, 8, (True, False))])
def test_requant_mixed_widths_same_containers(p_bits, q_bits, signs):
    """Activation and weight widths differ; output containers as wide as the input's, so the
    container-aligned slices are taken wherever the sums fit them (and the plan's otherwise)."""
    a_s, w_s = signs
    out_bits = p_bits
    for taps, rows, length in ((3, 3, 4099), (7, 2, 1000), (2, 5, 257)):
        rng = wl.rng_for("rq7", p_bits, q_bits, a_s, w_s, taps)
        x = wl.uniform_values(rng, (rows, length), p_bits, a_s)
        g = wl.uniform_values(rng, (taps,), q_bits, w_s)
        plan = requant_plan(p_bits, a_s, w_s, taps, out_bits, bits_w=q_bits)
        top = taps * ((1 << p_bits) - 1) * ((1 << q_bits) - 1)
        for mode in (hk.OUT_FULL, hk.OUT_VALID):
            for shift in (0, 1, max(0, int(top).bit_length() - out_bits - 1)):
                qmax = (1 << out_bits) - 1
                ref = oracle_requant(x, g, mode, shift, qmax, out_bits)
                out_len = length + taps - 1 if mode == hk.OUT_FULL else length - taps + 1
                row_bytes = hk.hikonv_bitdense_row_bytes(out_len, out_bits)
                out = Guarded(rows * row_bytes, torch.uint8, GUARD)
                hk.hikonv_conv1d_requant(plan, compact(x, p_bits), hk.FMT_BITDENSE, rows, length, dev(g), taps, mode,
                                         shift, qmax, out_bits, out.view)
                assert np.array_equal(out.result().reshape(rows, row_bytes), ref), (p_bits, q_bits, signs, taps, mode, shift)


def test_requant_refuses_aligned_plans_that_do_not_fit_the_call():
    """A container-aligned plan describes one kernel form; a call with another output container,
    or a plan whose slice width is not the one the operands take, is refused, nothing is written."""
    x, g = values("rq8", 4, False, False, 3, 2, 256)
    plan = hk.hikonv_plan_ex(bits_a=4, bits_w=4, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_CONV1D, taps=3,
                             objective=hk.OBJ_MEASURED_COST, out_bits=4)
    assert plan.stride_elems == 4
    out = Guarded(2 * 256, torch.uint8, GUARD)
    x_d, g_d = compact(x, 4), dev(g)
    with pytest.raises(hk.HikonvError) as e:    # 8-bit output containers with a plan made for 4-bit ones
        hk.hikonv_conv1d_requant(plan, x_d, hk.FMT_BITDENSE, 2, 256, g_d, 3, hk.OUT_VALID, 0, 15, 8, out.view)
    assert e.value.code == hk.EINVAL
    with pytest.raises(hk.HikonvError) as e:    # one value per byte in, 4-bit containers out
        hk.hikonv_conv1d_requant(plan, dev(x), hk.FMT_INT8, 2, 256, g_d, 3, hk.OUT_VALID, 0, 15, 4, out.view)
    assert e.value.code == hk.EINVAL
    with pytest.raises(hk.HikonvError) as e:    # int32 outputs take stride_elems = 1 plans only
        hk.hikonv_conv1d(plan, x_d, hk.FMT_BITDENSE, 2, 256, g_d, 3, hk.OUT_VALID, out.view)
    assert e.value.code == hk.EUNSUPPORTED
    out.result()


@pytest.mark.parametrize("bits,signed", [(5, False), (7, True), (8, False), (8, True)])
def test_requant_unpacked_windows_of_up_to_96_bits(bits, signed):
    """The baseline with 8-bit containers in and out and 6 or 7 taps reads its windows from four
    dwords: rows that end anywhere inside a window, short rows, both formats, both output modes."""
    for taps in (6, 7):
        for rows, length in ((3, 5), (4, 9), (2, 10), (5, 11), (3, 37), (2, 4099), (1, 20011), (6, 1023)):
            x, g = values("rq96", bits, signed, signed, taps, rows, length)
            for out_bits in (5, 8):
                qmax = (1 << out_bits) - 1 if out_bits < 8 else 255
                for mode in (hk.OUT_FULL, hk.OUT_VALID):
                    for shift in (0, pick_shift(bits, taps, out_bits)):
                        ref = oracle_requant(x, g, mode, shift, qmax, out_bits)
                        for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
                            got = run_requant(x, g, bits, signed, signed, mode, fmt, shift, qmax, out_bits, packed=False)
                            assert np.array_equal(got, ref), (bits, signed, taps, rows, length, out_bits, mode, shift, fmt)
