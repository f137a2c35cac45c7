"""GPU parity: 1-D convolution with in-kernel requantisation and bit-dense output through the
C ABI vs the oracle chain direct convolution -> ReLU/shift/clamp -> bit-dense packing,
byte for byte (padding bits of every row included)."""
import os

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import direct

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_00763_amd as hk
    from gpu_util import compact, conv1d_plan, dev

SIGNS = [(False, False), (True, True), (False, True), (True, False)]
GUARD = 0xA5


@pytest.fixture(autouse=True, params=["library_choice", "plan_slices"])
def requant_kernel(request):
    """Every case runs twice: with the library's own choice (container-aligned 16-bit slices where
    input and output containers are equal and the sums fit) and with the plan's N, K, S forced."""
    old = os.environ.get("HIKONV_REQUANT_KERNEL")
    if request.param == "plan_slices":
        os.environ["HIKONV_REQUANT_KERNEL"] = "1"
    else:
        os.environ.pop("HIKONV_REQUANT_KERNEL", None)
    yield request.param
    if old is None:
        os.environ.pop("HIKONV_REQUANT_KERNEL", None)
    else:
        os.environ["HIKONV_REQUANT_KERNEL"] = old


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
    q = torch.full((rows * row_bytes + 32,), GUARD, dtype=torch.uint8, device="cuda")
    x_d = compact(x, bits) if fmt == hk.FMT_BITDENSE else dev(x)
    g_d = dev(g)
    if packed:
        plan = conv1d_plan(bits, a_s, w_s, taps)
        hk.hikonv_conv1d_requant(plan, x_d, fmt, rows, length, g_d, taps, mode, shift, qmax, out_bits, q)
    else:
        hk.hikonv_conv1d_requant_unpacked(bits, bits, hk.signedness(a_s, w_s), x_d, fmt, rows, length, g_d, taps,
                                          mode, shift, qmax, out_bits, q)
    torch.cuda.synchronize()
    res = q.cpu().numpy()
    assert (res[rows * row_bytes:] == GUARD).all(), "wrote past the end of the output"
    return res[:rows * row_bytes].reshape(rows, row_bytes)


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


def test_requant_full_size_rows_sampled():
    """The benchmark's shape: 4096 x 65536, 3 taps, 4-bit unsigned in, 4-bit out; the oracle checks
    a sample of whole rows."""
    bits, taps, rows, length = 4, 3, 4096, 65536
    x, g = wl.conv1d_case(bits, False, taps, rows, length)
    shift, qmax, out_bits = 5, 15, 4
    x_d, g_d = compact(x, bits), dev(g)
    out_len = length + taps - 1
    row_bytes = hk.hikonv_bitdense_row_bytes(out_len, out_bits)
    sample = [0, 1, 2047, 4094, 4095] + list(wl.rng_for("rq_rows").integers(0, rows, 24))
    ref = oracle_requant(x[sample], g, hk.OUT_FULL, shift, qmax, out_bits)
    plan = conv1d_plan(bits, False, False, taps)
    for packed in (True, False):
        q = torch.full((rows * row_bytes + 32,), GUARD, dtype=torch.uint8, device="cuda")
        if packed:
            hk.hikonv_conv1d_requant(plan, x_d, hk.FMT_BITDENSE, rows, length, g_d, taps, hk.OUT_FULL, shift, qmax,
                                     out_bits, q)
        else:
            hk.hikonv_conv1d_requant_unpacked(bits, bits, 0, x_d, hk.FMT_BITDENSE, rows, length, g_d, taps,
                                              hk.OUT_FULL, shift, qmax, out_bits, q)
        torch.cuda.synchronize()
        assert (q[rows * row_bytes:] == GUARD).all()
        got = q[:rows * row_bytes].view(rows, row_bytes)[sample].cpu().numpy()
        assert np.array_equal(got, ref), packed


def test_requant_empty_and_rejected_arguments():
    x, g = values("rq4", 4, False, False, 3, 2, 64)
    plan = conv1d_plan(4, False, False, 3)
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
        plan = conv1d_plan(p_bits, a_s, w_s, taps, bits_w=q_bits)
        top = taps * ((1 << p_bits) - 1) * ((1 << q_bits) - 1)
        for mode in (hk.OUT_FULL, hk.OUT_VALID):
            for shift in (0, 1, max(0, int(top).bit_length() - out_bits - 1)):
                qmax = (1 << out_bits) - 1
                ref = oracle_requant(x, g, mode, shift, qmax, out_bits)
                out_len = length + taps - 1 if mode == hk.OUT_FULL else length - taps + 1
                row_bytes = hk.hikonv_bitdense_row_bytes(out_len, out_bits)
                q = torch.full((rows * row_bytes + 32,), GUARD, dtype=torch.uint8, device="cuda")
                hk.hikonv_conv1d_requant(plan, compact(x, p_bits), hk.FMT_BITDENSE, rows, length, dev(g), taps, mode,
                                         shift, qmax, out_bits, q)
                torch.cuda.synchronize()
                res = q.cpu().numpy()
                assert (res[rows * row_bytes:] == GUARD).all()
                assert np.array_equal(res[:rows * row_bytes].reshape(rows, row_bytes), ref), (p_bits, q_bits, signs, taps, mode, shift)
