"""GPU parity: packed and unpacked 1-D convolution through the C ABI vs the int64 oracle,
bit-exact, element by element."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_00763_amd as hk
    from gpu_util import run_conv1d, oracle_conv1d, conv1d_plan, dev, compact, Guarded, GUARD_I32

SIGNS = [(False, False), (True, True), (False, True), (True, False)]


@pytest.fixture(autouse=True, params=["library_choice", "lane_exchange"])
def kernel_form(request):
    """Every case runs on the kernel the library picks (a lane per aligned group of outputs where
    the plan allows it) and with the lane-per-block kernel asked for through the plan."""
    import gpu_util
    old = dict(gpu_util.CONV1D_DEFAULTS)
    gpu_util.CONV1D_DEFAULTS["kernel"] = hk.KERNEL_AUTO if request.param == "library_choice" else hk.KERNEL_LANES
    yield request.param
    gpu_util.CONV1D_DEFAULTS.update(old)


def test_lane_exchange_layout():
    out = torch.zeros(64, dtype=torch.int32, device="cuda")
    hk.hikonv_selftest_lane_shift(out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert got[0] == 0 and np.array_equal(got[1:], np.arange(100, 163))


@pytest.mark.parametrize("bits", range(1, 9))
@pytest.mark.parametrize("signs", SIGNS)
def test_conv1d_small_shapes(bits, signs):
    a_s, w_s = signs
    for taps in (1, 2, 3, 5, 7):
        for length in (1, 2, 6, 97, 1000):
            x, g = wl.conv1d_case(bits, a_s, taps, 3, length, tag="t1") if a_s == w_s else (
                wl.uniform_values(wl.rng_for("t1x", bits, taps, length), (3, length), bits, a_s),
                wl.uniform_values(wl.rng_for("t1g", bits, taps, length), (taps,), bits, w_s))
            for mode in (hk.OUT_FULL, hk.OUT_VALID):
                ref = oracle_conv1d(x, g, mode)
                for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
                    got = run_conv1d(x, g, bits, a_s, w_s, mode, fmt)
                    assert got.shape == ref.shape
                    assert np.array_equal(got, ref), (bits, signs, taps, length, mode, fmt)


@pytest.mark.parametrize("bits,signs,taps", [(1, (False, False), 3), (1, (True, True), 7), (2, (True, True), 3),
                                             (4, (False, False), 3), (4, (True, True), 5), (3, (False, True), 3),
                                             (6, (True, True), 3), (8, (False, False), 7), (8, (True, True), 3)])
def test_conv1d_several_tiles_and_ragged_tail(bits, signs, taps):
    a_s, w_s = signs
    rng = wl.rng_for("t2", bits, signs, taps)
    for rows, length in ((5, 20011), (2, 65536), (7, 4099)):
        x = wl.uniform_values(rng, (rows, length), bits, a_s)
        g = wl.uniform_values(rng, (taps,), bits, w_s)
        for mode in (hk.OUT_FULL, hk.OUT_VALID):
            ref = oracle_conv1d(x, g, mode)
            for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
                assert np.array_equal(run_conv1d(x, g, bits, a_s, w_s, mode, fmt), ref)
            assert np.array_equal(run_conv1d(x, g, bits, a_s, w_s, mode, hk.FMT_BITDENSE, packed=False), ref)


@pytest.mark.parametrize("bits,signed", [(1, False), (2, True), (4, False), (4, True), (8, True)])
def test_conv1d_extreme_values(bits, signed):
    lo, hi = wl.value_range(bits, signed)
    dt = np.int8 if signed else np.uint8
    for taps in (3, 7):
        for fv in (lo, hi):
            for gv in (lo, hi):
                x = np.full((2, 3001), fv, dtype=dt)
                g = np.full((taps,), gv, dtype=dt)
                ref = oracle_conv1d(x, g, hk.OUT_FULL)
                assert np.array_equal(run_conv1d(x, g, bits, signed, signed, hk.OUT_FULL, hk.FMT_BITDENSE), ref)


def test_conv1d_config1():
    x, g = wl.config1()
    ref = oracle_conv1d(x, g, hk.OUT_VALID)
    assert ref.shape == (1, 4094)
    plan = conv1d_plan(4, False, False, 3)
    assert (plan.N, plan.K, plan.S, plan.G_b) == (3, 3, 10, 2)
    for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
        assert np.array_equal(run_conv1d(x, g, 4, False, False, hk.OUT_VALID, fmt), ref)
        assert np.array_equal(run_conv1d(x, g, 4, False, False, hk.OUT_VALID, fmt, packed=False), ref)


def test_conv1d_unpacked_small():
    for bits, signs in ((1, (False, False)), (4, (True, True)), (8, (False, True)), (5, (True, False))):
        a_s, w_s = signs
        rng = wl.rng_for("t3", bits, signs)
        for taps, length in ((1, 9), (3, 130), (7, 1025), (5, 3)):
            x = wl.uniform_values(rng, (4, length), bits, a_s)
            g = wl.uniform_values(rng, (taps,), bits, w_s)
            for mode in (hk.OUT_FULL, hk.OUT_VALID):
                ref = oracle_conv1d(x, g, mode)
                for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
                    assert np.array_equal(run_conv1d(x, g, bits, a_s, w_s, mode, fmt, packed=False), ref)


def test_conv1d_empty_and_error_paths():
    plan = conv1d_plan(4, False, False, 3)
    y = torch.zeros(16, dtype=torch.int32, device="cuda")
    x = torch.zeros(16, dtype=torch.uint8, device="cuda")
    g = torch.zeros(3, dtype=torch.uint8, device="cuda")
    hk.hikonv_conv1d(plan, x, hk.FMT_INT8, 0, 10, g, 3, hk.OUT_FULL, y)          # no rows: ok
    hk.hikonv_conv1d(plan, x, hk.FMT_INT8, 2, 2, g, 3, hk.OUT_VALID, y)          # len < taps, valid: ok
    with pytest.raises(hk.HikonvError) as e:
        hk.hikonv_conv1d(plan, x, hk.FMT_INT8, 1, 10, g, 5, hk.OUT_FULL, y)      # taps differ from the plan
    assert e.value.code == hk.EINVAL
    with pytest.raises(hk.HikonvError) as e:
        hk.hikonv_conv1d(plan, None, hk.FMT_INT8, 1, 10, g, 3, hk.OUT_FULL, y)
    assert e.value.code == hk.EINVAL
    with pytest.raises(hk.HikonvError) as e:
        hk.hikonv_conv1d(plan, x, 7, 1, 10, g, 3, hk.OUT_FULL, y)
    assert e.value.code == hk.EINVAL
    torch.cuda.synchronize()


def _first_mismatch(got_d, ref_d, out_len):
    bad = torch.nonzero(got_d != ref_d)[0].item()
    return "row %d, output %d: got %d, oracle %d" % (bad // out_len, bad % out_len, got_d[bad].item(), ref_d[bad].item())


@pytest.mark.parametrize("signed", [False, True])
@pytest.mark.parametrize("bits", range(1, 9))
def test_conv1d_full_size_sweep_all_rows(bits, signed):
    """All 48 cases of the sweep at 4096 x 65536 in the launch configuration the benchmark times
    (bit-dense input, valid outputs, 256-byte aligned y): every one of the 4096 x out_len
    outputs of the packed kernel, and of the unpacked baseline, is compared with the oracle's
    (on the device, so that no second copy of the outputs crosses to the host)."""
    rows, length = 4096, 65536
    x = wl.uniform_values(wl.rng_for("c2x", bits, signed), (rows, length), bits, signed)
    x_d = compact(x, bits)
    for taps in (3, 5, 7):
        g = wl.uniform_values(wl.rng_for("c2g", bits, signed, taps), (taps,), bits, signed)
        plan = conv1d_plan(bits, signed, signed, taps)
        out_len = length - taps + 1
        ref_d = torch.from_numpy(oracle_conv1d(x, g, hk.OUT_VALID)).cuda().view(-1)
        out = Guarded(rows * out_len)
        hk.hikonv_conv1d(plan, x_d, hk.FMT_BITDENSE, rows, length, dev(g), taps, hk.OUT_VALID, out.view)
        torch.cuda.synchronize()
        out.check()
        assert torch.equal(out.view, ref_d), (bits, signed, taps, _first_mismatch(out.view, ref_d, out_len))
        out.view.fill_(GUARD_I32)
        hk.hikonv_conv1d_unpacked(bits, bits, hk.signedness(signed, signed), x_d, hk.FMT_BITDENSE, rows, length,
                                  dev(g), taps, hk.OUT_VALID, out.view)
        torch.cuda.synchronize()
        out.check()
        assert torch.equal(out.view, ref_d), ("unpacked", bits, signed, taps, _first_mismatch(out.view, ref_d, out_len))
        del out, ref_d


def _phase_plans():
    """One plan of every form of the streaming kernel: single B word (N = 11, 6, 3), taps cut into
    chunks of N taps whose delayed words come from the preceding lanes (2, 3 and 4 chunks), and
    chunks cut out of one 64-bit window."""
    return [(1, False, 3), (2, False, 3), (4, False, 3), (4, True, 3),     # one B word: N = 11, 6, 3
            (8, False, 3), (8, True, 7), (6, True, 7),                      # K = N chunks shared through the lanes
            (3, False, 5), (2, True, 7), (5, False, 7)]                     # other chunked plans


@pytest.mark.parametrize("bits,signed,taps", _phase_plans() if torch.cuda.is_available() else [])
def test_conv1d_every_store_phase(bits, signed, taps):
    """The streaming kernel cuts a row's outputs into runs whose ends fall on 128-byte lines of y;
    where they fall depends on (address of y / 4 + row * out_len) mod 32.  Walk every reachable
    value: y moved off its alignment by 0, 4, ..., 28 outputs, out_len mod 32 over 0..31, five
    rows of several runs each; guard regions on both sides of y."""
    plan = conv1d_plan(bits, signed, signed, taps)
    seen = set()
    for extra in range(32):
        length = 3 * 1536 + 7 + extra                                # three to four runs per row
        x = wl.uniform_values(wl.rng_for("ph", bits, signed, taps, extra), (5, length), bits, signed)
        g = wl.uniform_values(wl.rng_for("phg", bits, signed, taps), (taps,), bits, signed)
        for mode in (hk.OUT_VALID, hk.OUT_FULL):
            ref = oracle_conv1d(x, g, mode)
            for y_offset in range(0, 32, 4):
                got = run_conv1d(x, g, bits, signed, signed, mode, hk.FMT_BITDENSE, plan=plan, y_offset=y_offset)
                assert np.array_equal(got, ref), (bits, signed, taps, length, mode, y_offset)
                seen.update((y_offset + r * ref.shape[1]) % 32 for r in range(5))
            got = run_conv1d(x, g, bits, signed, signed, mode, hk.FMT_BITDENSE, packed=False, y_offset=4 * (extra % 8))
            assert np.array_equal(got, ref), ("unpacked", bits, signed, taps, length, mode)
    assert seen == set(range(32))


@pytest.mark.parametrize("bits,signed", [(1, False), (2, True), (4, False), (4, True), (8, False)])
def test_conv1d_every_length_around_group_boundaries(bits, signed):
    """Rows so short that a lane's group of eight (four) outputs is never complete, rows that end
    anywhere inside a group or a 128-byte line, several rows so that the groups start at every
    offset: packed and unpacked kernels, both output modes."""
    lengths = list(range(1, 41)) + [47, 48, 49, 63, 64, 65, 71, 72, 73, 127, 128, 129, 255, 256, 257, 511, 513]
    for taps in (1, 3, 7):
        g = wl.uniform_values(wl.rng_for("lb-g", bits, signed, taps), (taps,), bits, signed)
        for length in lengths:
            x = wl.uniform_values(wl.rng_for("lb", bits, signed, taps, length), (4, length), bits, signed)
            for mode in (hk.OUT_FULL, hk.OUT_VALID):
                ref = oracle_conv1d(x, g, mode)
                got = run_conv1d(x, g, bits, signed, signed, mode, hk.FMT_BITDENSE, y_offset=4 * (length % 8))
                assert np.array_equal(got, ref), (bits, signed, taps, length, mode)
                got = run_conv1d(x, g, bits, signed, signed, mode, hk.FMT_BITDENSE, packed=False)
                assert np.array_equal(got, ref), ("unpacked", bits, signed, taps, length, mode)


def test_conv1d_many_short_rows_and_one_long_row():
    # more rows than a grid dimension holds; rows shorter than one packed run; one very long row
    for bits, signed, taps in ((4, False, 3), (1, True, 7), (8, True, 3)):
        for rows, length in ((70001, 37), (1, (1 << 22) + 5), (3, 1513 * 3)):
            x = wl.uniform_values(wl.rng_for("t5", bits, signed, rows), (rows, length), bits, signed)
            g = wl.uniform_values(wl.rng_for("t5g", bits, signed, taps), (taps,), bits, signed)
            for mode in (hk.OUT_VALID, hk.OUT_FULL):
                ref = oracle_conv1d(x, g, mode)
                assert np.array_equal(run_conv1d(x, g, bits, signed, signed, mode, hk.FMT_BITDENSE), ref)
                assert np.array_equal(run_conv1d(x, g, bits, signed, signed, mode, hk.FMT_INT8, packed=False), ref)


def test_conv1d_int8_rows_that_do_not_fill_dwords():
    # one value per byte, odd row length: rows start at any byte offset and the buffer ends mid-dword
    for bits, signed in ((4, True), (7, False), (2, False)):
        for rows, length in ((5, 1001), (3, 7), (2, 4099)):
            x = wl.uniform_values(wl.rng_for("t6", bits, signed, rows, length), (rows, length), bits, signed)
            g = wl.uniform_values(wl.rng_for("t6g", bits, signed), (3,), bits, signed)
            for mode in (hk.OUT_VALID, hk.OUT_FULL):
                ref = oracle_conv1d(x, g, mode)
                assert np.array_equal(run_conv1d(x, g, bits, signed, signed, mode, hk.FMT_INT8), ref)
                assert np.array_equal(run_conv1d(x, g, bits, signed, signed, mode, hk.FMT_INT8, packed=False), ref)
