"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares,
and its host-side planner agrees with the paper's model (oracle/plan_model.py) and with the
big-integer packed model on the corner inputs that decide exactness."""
import itertools
import os
import re

import numpy as np
import pytest

import paper_2208_00763_amd as hk
from oracle import packed_model as pm, plan_model as pl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "hikonv.h")).read() + open(os.path.join(ROOT, "include", "hikonv_bench.h")).read()
    declared = set(re.findall(r"\b(hikonv_[a-z0-9_]+)\s*\(", header))
    declared -= {"hikonv_plan_t"}
    assert len(declared) >= 18
    for name in declared:
        assert hasattr(hk.lib, name), name
    assert declared == set(hk.SIGNATURES), declared ^ set(hk.SIGNATURES)


def test_strerror_and_codes():
    assert hk.hikonv_strerror(0) == "ok"
    for code in range(-7, 0):
        assert hk.hikonv_strerror(code) not in ("ok", "unknown error")
    assert hk.hikonv_strerror(-99) == "unknown error"


def test_bitdense_row_bytes():
    assert hk.hikonv_bitdense_row_bytes(65536, 4) == 32768
    assert hk.hikonv_bitdense_row_bytes(65536, 1) == 8192
    assert hk.hikonv_bitdense_row_bytes(9, 1) == 4 and hk.hikonv_bitdense_row_bytes(0, 3) == 0
    assert hk.hikonv_bitdense_row_bytes(10, 9) < 0


@pytest.mark.parametrize("widths", [(27, 18), (32, 32), (24, 24), (64, 64)])
def test_single_mode_unsigned_plans_equal_the_paper_model(widths):
    l_a, l_b = widths
    for p, q in itertools.product(range(1, 9), repeat=2):
        got = hk.hikonv_plan_ex(bits_a=p, bits_w=q, L_A=l_a, L_B=l_b, mode=hk.MODE_SINGLE)
        ref = pl.paper_search(p, q, l_a, l_b, pl.SINGLE)
        assert (got.N, got.K, got.S, got.G_b, got.ops_per_mul) == (ref["N"], ref["K"], ref["S"], ref["G_b"], ref["ops"])
        assert got.paper_exact == 1


def test_headline_entry_point():
    assert [hk.hikonv_plan(b, b, 0, 32).ops_per_mul for b in range(1, 9)] == [113, 41, 25, 13, 13, 8, 5, 5]
    p = hk.hikonv_plan(4, 4, 0, 32)
    assert (p.N, p.K, p.S, p.G_b, p.L_acc, p.mode) == (3, 3, 10, 2, 64, hk.MODE_SINGLE)


@pytest.mark.parametrize("taps", [1, 2, 3, 5, 7])
def test_conv1d_plans_unsigned_equal_the_paper_model(taps):
    for b in range(1, 9):
        got = hk.hikonv_plan_ex(bits_a=b, bits_w=b, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_CONV1D, taps=taps)
        ref = pl.paper_search_taps(b, b, 32, 32, taps, pl.CONV1D)
        assert (got.N, got.K, got.S, got.G_b, got.chunks) == (ref["N"], ref["K"], ref["S"], ref["G_b"], ref["chunks"])
        assert got.paper_exact == 1 and got.K <= got.N + 1


def _corner_inputs(plan, length):
    ra = (-(1 << (plan.bits_a - 1)), (1 << (plan.bits_a - 1)) - 1) if plan.a_signed else (0, (1 << plan.bits_a) - 1)
    rw = (-(1 << (plan.bits_w - 1)), (1 << (plan.bits_w - 1)) - 1) if plan.w_signed else (0, (1 << plan.bits_w) - 1)
    for fa in ra:
        for gw in rw:
            yield [fa] * length, [gw] * plan.taps


@pytest.mark.parametrize("tight", [0, 1])
@pytest.mark.parametrize("signs", [(1, 1), (0, 1), (1, 0)])
@pytest.mark.parametrize("taps", [3, 5, 7])
def test_signed_conv1d_plans_are_exact_on_corners(signs, taps, tight):
    for b in range(1, 9):
        plan = hk.hikonv_plan_ex(bits_a=b, bits_w=b, a_signed=signs[0], w_signed=signs[1], L_A=32, L_B=32, L_acc=64,
                                 mode=hk.MODE_CONV1D, taps=taps, tight=tight)
        assert hk.hikonv_plan_check(plan) == hk.OK
        for f, g in _corner_inputs(plan, 4 * plan.N + 1):
            # operands must fit the signed 32-bit multiplier inputs
            a_word = pm.pack(f[:plan.N], plan.S)
            assert -2 ** 31 <= a_word < 2 ** 31
            for c0 in range(0, taps, plan.K):
                assert -2 ** 31 <= pm.pack(g[c0:c0 + plan.K], plan.S) < 2 ** 31
            assert pm.conv1d_packed(f, g, plan.N, plan.K, plan.S, True) == np.convolve(f, g).tolist()
        ref = pl.paper_search_taps(b, b, 32, 32, taps, pl.CONV1D)
        same = (plan.N, plan.K, plan.S) == (ref["N"], ref["K"], ref["S"])
        assert bool(plan.paper_exact) == same


def test_paper_plans_that_are_one_bit_short_are_rejected():
    # (i) signed 1-bit values {-1,0}: eight products of (-1)(-1) reach 2^(S-1) for the printed S=4
    p = hk.hikonv_plan(1, 1, hk.A_SIGNED | hk.W_SIGNED, 32)
    ref = pl.paper_search(1, 1, 32, 32, pl.SINGLE)
    assert p.paper_exact == 0 and (ref["N"], ref["K"], ref["S"]) == (8, 8, 4)
    bad = hk.Plan(**{**p.as_dict(), "N": 8, "K": 8, "S": 4, "G_b": 3})
    assert hk.hikonv_plan_check(bad) == hk.EOVERFLOW
    assert pm.fnk([-1] * 8, [-1] * 8, 4, True)[0] != np.convolve([-1] * 8, [-1] * 8).tolist()
    assert pm.fnk([-1] * p.N, [-1] * p.K, p.S, True)[0] == np.convolve([-1] * p.N, [-1] * p.K).tolist()
    # (ii) the signed packed word of all-minimum inputs needs one bit more than Eq. (slice2) counts:
    # 2-bit signed, K=3 in 1-D mode: the printed N=6, S=6 fills 32 bits exactly
    bad = hk.hikonv_plan_ex(bits_a=2, bits_w=2, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_CONV1D, taps=3)
    assert (bad.N, bad.S) == (6, 6)
    bad.a_signed = bad.w_signed = 1
    assert hk.hikonv_plan_check(bad) == hk.EOVERFLOW
    assert pm.pack([-2] * 6, 6) < -2 ** 31
    good = hk.hikonv_plan_ex(bits_a=2, bits_w=2, a_signed=1, w_signed=1, L_A=32, L_B=32, L_acc=64,
                             mode=hk.MODE_CONV1D, taps=3)
    assert (good.N, good.S, good.paper_exact) == (5, 6, 0)
    # 6-bit signed on a single 32x32 multiplier: N=3, S=13 fills 32 bits exactly
    ref = pl.paper_search(6, 6, 32, 32, pl.SINGLE)
    p6 = hk.hikonv_plan(6, 6, 3, 32)
    assert (ref["N"], ref["S"]) == (3, 13) and pm.pack([-32] * 3, 13) < -2 ** 31
    assert hk.hikonv_plan_check(p6) == hk.OK and -2 ** 31 <= pm.pack([-32] * p6.N, p6.S)


def test_tight_plans_use_the_smallest_exact_slice():
    """Beyond Eq. (slice1): the slice only has to hold the largest segment sum of the declared
    ranges.  Three signed 4-bit products reach 192 in magnitude: 9 bits instead of 4+4+2."""
    loose = hk.hikonv_plan_ex(bits_a=4, bits_w=4, a_signed=1, w_signed=1, L_A=32, L_B=32, L_acc=64,
                              mode=hk.MODE_CONV1D, taps=3)
    tight = hk.hikonv_plan_ex(bits_a=4, bits_w=4, a_signed=1, w_signed=1, L_A=32, L_B=32, L_acc=64,
                              mode=hk.MODE_CONV1D, taps=3, tight=1)
    assert (loose.N, loose.S, loose.ops_per_mul, loose.paper_exact) == (3, 10, 13, 1)
    assert (tight.N, tight.S, tight.ops_per_mul, tight.paper_exact) == (4, 9, 18, 0)
    # one bit less is inexact, and the planner's check says so
    short = hk.Plan(**{**tight.as_dict(), "S": 8})
    assert hk.hikonv_plan_check(short) == hk.EOVERFLOW
    f, g = [-8] * 9, [-8] * 3
    assert pm.conv1d_packed(f, g, 4, 3, 9, True) == np.convolve(f, g).tolist()
    assert pm.conv1d_packed(f, g, 4, 3, 8, True) != np.convolve(f, g).tolist()
    # 1-bit unsigned, 3 taps: sums reach 3, two bits suffice; 16 values per 32-bit word
    t1 = hk.hikonv_plan_ex(bits_a=1, bits_w=1, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_CONV1D, taps=3, tight=1)
    assert (t1.N, t1.S) == (16, 2)
    # a tight plan is never worse than the default one, for every width and signedness
    for b in range(1, 9):
        for sa, sw in ((0, 0), (1, 1), (0, 1), (1, 0)):
            for taps in (1, 3, 5, 7):
                kw = dict(bits_a=b, bits_w=b, a_signed=sa, w_signed=sw, L_A=32, L_B=32, L_acc=64,
                          mode=hk.MODE_CONV1D, taps=taps)
                d, t = hk.hikonv_plan_ex(**kw), hk.hikonv_plan_ex(tight=1, **kw)
                assert t.N * d.chunks >= d.N * t.chunks and hk.hikonv_plan_check(t) == hk.OK
                if (t.N, t.K) == (d.N, d.K):
                    assert t.S <= d.S
                less = hk.Plan(**{**t.as_dict(), "S": t.S - 1})
                assert t.S == 1 or hk.hikonv_plan_check(less) != hk.OK


@pytest.mark.parametrize("tight", [0, 1])
@pytest.mark.parametrize("wide", [True, False])
def test_dnn_plans_are_exact_on_corners(wide, tight):
    width, acc = (32, 64) if wide else (24, 32)
    for b, sa, sw in ((1, 0, 0), (2, 1, 1), (4, 1, 1), (4, 0, 1), (4, 0, 0), (8, 1, 1), (3, 0, 1)):
        for taps in (1, 3, 5):
            for m in (1, 2, 5, 9, 0):
                try:
                    plan = hk.hikonv_plan_ex(bits_a=b, bits_w=b, a_signed=sa, w_signed=sw, L_A=width, L_B=width,
                                             L_acc=acc, mode=hk.MODE_DNN, M=m, taps=taps, tight=tight)
                except hk.HikonvError as e:
                    assert e.code == hk.ENOPLAN
                    continue
                assert hk.hikonv_plan_check(plan) == hk.OK and plan.K <= plan.N + 1
                signed = bool(sa or sw)
                ra = (-(1 << (b - 1)), (1 << (b - 1)) - 1) if sa else (0, (1 << b) - 1)
                rw = (-(1 << (b - 1)), (1 << (b - 1)) - 1) if sw else (0, (1 << b) - 1)
                c_in = plan.M if tight else min(plan.M, 40)   # one split group of channels, one kernel row
                for fa, gw in itertools.product(ra, rw):
                    x = [[[fa] * (2 * plan.N + 1)] for _ in range(c_in)]
                    w = [[[[gw] * taps] for _ in range(c_in)]]
                    got = pm.conv2d_packed(x, w, taps - 1, plan.N, plan.K, plan.S, plan.M, signed)
                    row = np.convolve([fa] * (2 * plan.N + 1), [gw] * taps) * c_in
                    assert got[0][taps - 1] == row.tolist()   # output row aligned with the only input row
                    # accumulated word fits the accumulator register (top segment included)
                    a_word = pm.pack([fa] * plan.N, plan.S)
                    total = sum(a_word * pm.pack([gw] * min(plan.K, taps - c0), plan.S)
                                for c0 in range(0, taps, plan.K)) * plan.M
                    if signed:
                        assert -2 ** (acc - 1) <= total < 2 ** (acc - 1)
                    else:
                        assert 0 <= total < 2 ** acc


def test_bad_requests():
    for kw in (dict(bits_a=0, bits_w=4), dict(bits_a=4, bits_w=9), dict(bits_a=4, bits_w=4, L_A=0),
               dict(bits_a=4, bits_w=4, mode=7), dict(bits_a=2, bits_w=1, bipolar=1)):
        base = dict(L_A=32, L_B=32, mode=hk.MODE_SINGLE)
        base.update(kw)
        with pytest.raises(hk.HikonvError) as e:
            hk.hikonv_plan_ex(**base)
        assert e.value.code == hk.EINVAL
    with pytest.raises(hk.HikonvError) as e:
        hk.hikonv_plan_ex(bits_a=8, bits_w=8, L_A=8, L_B=8, L_acc=8, mode=hk.MODE_SINGLE)
    assert e.value.code == hk.ENOPLAN
    assert hk.lib.hikonv_plan(4, 4, 0, 32, None) == hk.EINVAL


# ---- argument checks of the device entry points (they fail before any launch) -------------
class _Fake:
    """Stands in for a device tensor: the checks below reject the call before it is touched."""
    def __init__(self, addr, nbytes=1 << 20):
        self._addr, self._n = addr, nbytes

    def data_ptr(self):
        return self._addr

    def numel(self):
        return self._n

    def element_size(self):
        return 1


def _dnn_plan(**kw):
    base = dict(bits_a=4, bits_w=4, a_signed=1, w_signed=1, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_DNN, M=5, taps=3)
    base.update(kw)
    return hk.hikonv_plan_ex(**base)


def test_conv2d_argument_checks():
    plan = _dnn_plan()
    x, w, y, ws = _Fake(0x1000), _Fake(0x2000), _Fake(0x3000), _Fake(0x10000)
    args = (hk.FMT_INT8, 1, 8, 10, 10)

    def code(fn):
        with pytest.raises(hk.HikonvError) as e:
            fn()
        return e.value.code

    # kernel width differs from the plan's taps
    assert code(lambda: hk.hikonv_conv2d(plan, x, *args, w, 8, 3, 5, 1, 1, ws, y, stream=0)) == hk.EINVAL
    # padding wider than the kernel allows
    assert code(lambda: hk.hikonv_conv2d(plan, x, *args, w, 8, 3, 3, 1, 3, ws, y, stream=0)) == hk.EUNSUPPORTED
    # kernel larger than the padded image
    assert code(lambda: hk.hikonv_conv2d(plan, x, hk.FMT_INT8, 1, 8, 1, 1, w, 8, 3, 3, 1, 0, ws, y, stream=0)) == hk.EINVAL
    # workspace too small / misaligned / missing
    assert code(lambda: hk.hikonv_conv2d(plan, x, *args, w, 8, 3, 3, 1, 1, _Fake(0x10000, 16), y, stream=0)) == hk.EWORKSPACE
    assert code(lambda: hk.hikonv_conv2d(plan, x, *args, w, 8, 3, 3, 1, 1, _Fake(0x10004), y, stream=0)) == hk.EWORKSPACE
    # null tensors, bad format
    assert code(lambda: hk.hikonv_conv2d(plan, None, *args, w, 8, 3, 3, 1, 1, ws, y, stream=0)) == hk.EINVAL
    assert code(lambda: hk.hikonv_conv2d(plan, x, 9, 1, 8, 10, 10, w, 8, 3, 3, 1, 1, ws, y, stream=0)) == hk.EINVAL
    # a 1-D plan is not a layer plan
    p1 = hk.hikonv_plan_ex(bits_a=4, bits_w=4, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_CONV1D, taps=3)
    assert code(lambda: hk.hikonv_conv2d(p1, x, *args, w, 8, 3, 3, 1, 1, ws, y, stream=0)) == hk.EINVAL
    # int32 overflow of the worst-case sum: 8-bit unsigned, 40000 channels of 3x3
    p8 = _dnn_plan(bits_a=8, bits_w=8, a_signed=0, w_signed=0, M=1)
    assert code(lambda: hk.hikonv_conv2d(p8, x, hk.FMT_INT8, 1, 40000, 10, 10, w, 8, 3, 3, 1, 1, ws, y, stream=0)) == hk.EOVERFLOW
    # a plan edited so that its fields overflow is refused
    bad = hk.Plan(**{**plan.as_dict(), "S": plan.S - 3})
    assert code(lambda: hk.hikonv_conv2d(bad, x, *args, w, 8, 3, 3, 1, 1, ws, y, stream=0)) == hk.EOVERFLOW
    # unsupported multiplier width
    p64 = hk.Plan(**{**plan.as_dict(), "L_A": 64, "L_B": 64, "L_acc": 128})
    assert code(lambda: hk.hikonv_conv2d(p64, x, *args, w, 8, 3, 3, 1, 1, ws, y, stream=0)) == hk.EUNSUPPORTED


def test_strided_and_3d_argument_checks():
    plan3 = _dnn_plan()                                   # taps = 3
    plan2 = _dnn_plan(taps=2)                             # ceil(3/2): the polyphase form of a 3-tap row at stride 2
    x, w, y, ws = _Fake(0x1000), _Fake(0x2000), _Fake(0x3000), _Fake(0x100000)

    def code(fn):
        with pytest.raises(hk.HikonvError) as e:
            fn()
        return e.value.code

    # which tap counts a strided layer accepts: Kw (every column computed) or ceil(Kw/stride) (polyphase)
    assert hk.hikonv_conv2d_workspace_bytes(plan3, 1, 8, 10, 10, 8, 3, 3, 2, 1, True) > 0
    assert hk.hikonv_conv2d_workspace_bytes(plan2, 1, 8, 10, 10, 8, 3, 3, 2, 1, True) > 0
    assert hk.hikonv_conv2d_workspace_bytes(plan2, 1, 8, 10, 10, 8, 3, 3, 1, 1, True) == 0
    assert hk.hikonv_conv2d_workspace_bytes(plan2, 1, 8, 10, 10, 8, 3, 5, 2, 1, True) == 0
    assert code(lambda: hk.hikonv_conv2d(plan2, x, hk.FMT_INT8, 1, 8, 10, 10, w, 8, 3, 3, 3, 1, ws, y, stream=0)) == hk.EINVAL
    # polyphase packs `stride` phases per channel: more packed channels, narrower rows, any padding
    # (one B word per term and channel, 8 channels per group, plus one group of read-ahead slack, rounded to 256)
    assert hk.hikonv_packed_weights_bytes_ex(plan3, 8, 8, 1, 3, 3, 2) == 8 * 3 * 32 + 256
    assert hk.hikonv_packed_weights_bytes_ex(plan2, 8, 8, 1, 3, 3, 2) == 2 * 8 * 3 * 32 + 256
    assert hk.hikonv_packed_weights_bytes_ex(plan2, 8, 8, 1, 3, 3, 1) == 0
    assert hk.hikonv_conv2d_workspace_bytes(plan2, 1, 8, 10, 10, 8, 3, 3, 2, 4, True) > 0       # pad > Kw-1 is fine here
    assert hk.hikonv_conv2d_workspace_bytes(plan3, 1, 8, 10, 10, 8, 3, 3, 2, 4, True) == 0
    # 3-D: workspace grows with the padded depth, kernel depth must fit, no pre-packed activations
    ws1 = hk.hikonv_conv3d_workspace_bytes(plan3, 1, 8, 4, 10, 10, 8, 3, 3, 3, 1, 1, True)
    ws2 = hk.hikonv_conv3d_workspace_bytes(plan3, 1, 8, 10, 10, 10, 8, 3, 3, 3, 1, 1, True)
    assert 0 < ws1 < ws2
    assert hk.hikonv_conv3d_workspace_bytes(plan3, 1, 8, 1, 10, 10, 8, 5, 3, 3, 1, 1, True) == 0   # depth 1 + 2 < 5
    assert hk.hikonv_packed_weights_bytes_ex(plan3, 8, 8, 3, 3, 3, 1) == 3 * 8 * 3 * 32 + 256
    args3 = (1, 8, 4, 10, 10)
    assert code(lambda: hk.hikonv_conv3d(plan3, x, hk.FMT_PACKED, *args3, w, False, 8, 3, 3, 3, 1, 1, ws, y, stream=0)) == hk.EINVAL
    assert code(lambda: hk.hikonv_conv3d(plan3, None, hk.FMT_INT8, *args3, w, False, 8, 3, 3, 3, 1, 1, ws, y, stream=0)) == hk.EINVAL
    assert code(lambda: hk.hikonv_conv3d(plan3, x, hk.FMT_INT8, *args3, w, False, 8, 3, 3, 3, 1, 1, _Fake(0x100000, 64), y, stream=0)) == hk.EWORKSPACE
    assert code(lambda: hk.hikonv_conv3d(plan3, x, hk.FMT_INT8, 1, 8, 0, 10, 10, w, False, 8, 3, 3, 3, 1, 1, ws, y, stream=0)) == hk.EINVAL
    assert code(lambda: hk.hikonv_pack_weights_ex(plan3, w, 8, 8, 3, 3, 3, 1, _Fake(0x100010), stream=0)) == hk.EINVAL   # alignment
    # the fused epilogue writes one column phase only
    nxt = _dnn_plan(bits_a=4, bits_w=4, a_signed=0, w_signed=1, taps=2)
    assert code(lambda: hk.hikonv_epilogue_pack(x, 1, 8, 10, 10, 3, 15, False, nxt, 8, 3, 3, 2, 1, ws, stream=0)) == hk.EUNSUPPORTED


def test_workspace_and_packed_weight_sizes():
    plan = _dnn_plan()
    ws = hk.hikonv_conv2d_workspace_bytes(plan, 1, 64, 56, 56, 64, 3, 3, 1, 1, True)
    ws_raw = hk.hikonv_conv2d_workspace_bytes(plan, 1, 64, 56, 56, 64, 3, 3, 1, 1, False)
    pw = hk.hikonv_packed_weights_bytes(plan, 64, 64, 3, 3)
    assert ws % 256 == 0 and pw % 256 == 0 and ws_raw == ws + pw
    # packed activations: chunks * N * C * (H+2p) * (ceil((W+p)/N)+1) words
    assert ws >= 64 * 58 * (19 + 1) * 4 and pw >= 8 * 64 * 3 * 8 * 4
    assert hk.hikonv_conv2d_workspace_bytes(plan, 1, 64, 56, 56, 64, 3, 5, 1, 1, True) == 0   # taps differ from the plan
    bip = hk.hikonv_plan_ex(bits_a=1, bits_w=1, bipolar=1, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_DNN, M=0, taps=3)
    # {-1,+1} layers are ordinary signed layers (values travel as signed slices): one B word per term, no extra tables
    assert hk.hikonv_packed_weights_bytes(bip, 256, 256, 3, 3) == 32 * 768 * 8 * 4 + 256
    assert (bip.N, bip.K, bip.S, bip.M) == (4, 3, 10, 170) and hk.hikonv_plan_check(bip) == hk.OK


def test_conv1d_and_misc_argument_checks():
    plan = hk.hikonv_plan_ex(bits_a=4, bits_w=4, L_A=32, L_B=32, L_acc=64, mode=hk.MODE_CONV1D, taps=3)
    x, g, y = _Fake(0x1000), _Fake(0x2000), _Fake(0x3000)

    def code(fn):
        with pytest.raises(hk.HikonvError) as e:
            fn()
        return e.value.code

    assert code(lambda: hk.hikonv_conv1d(plan, x, hk.FMT_INT8, 2, 100, g, 3, 5, y, stream=0)) == hk.EINVAL        # out mode
    assert code(lambda: hk.hikonv_conv1d(plan, x, hk.FMT_INT8, -1, 100, g, 3, hk.OUT_FULL, y, stream=0)) == hk.EINVAL
    assert code(lambda: hk.hikonv_conv1d(plan, _Fake(0x1002), hk.FMT_INT8, 2, 100, g, 3, hk.OUT_FULL, y, stream=0)) == hk.EINVAL  # x alignment
    assert code(lambda: hk.hikonv_conv1d(plan, x, hk.FMT_INT8, 2, 100, g, 3, hk.OUT_FULL, _Fake(0x3004), stream=0)) == hk.EINVAL  # y alignment
    bip = hk.Plan(**{**plan.as_dict(), "bipolar": 1, "bits_a": 1, "bits_w": 1})
    assert code(lambda: hk.hikonv_conv1d(bip, x, hk.FMT_INT8, 2, 100, g, 3, hk.OUT_FULL, y, stream=0)) == hk.EUNSUPPORTED
    narrow = hk.Plan(**{**plan.as_dict(), "L_A": 24, "L_B": 24, "L_acc": 32})
    assert code(lambda: hk.hikonv_conv1d(narrow, x, hk.FMT_INT8, 2, 100, g, 3, hk.OUT_FULL, y, stream=0)) == hk.EUNSUPPORTED
    assert code(lambda: hk.hikonv_compact(x, 2, 100, 9, False, y, stream=0)) == hk.EINVAL
    assert code(lambda: hk.hikonv_compact(x, 2, 100, 4, True, y, stream=0)) == hk.EINVAL                          # bipolar needs 1 bit
    assert code(lambda: hk.hikonv_check_range(x, 100, 0, False, False, y, stream=0)) == hk.EINVAL
    assert code(lambda: hk.hikonv_check_range(x, 100, 4, False, True, y, stream=0)) == hk.EINVAL                  # bipolar needs 1 bit
    assert code(lambda: hk.hikonv_check_range(x, 100, 4, False, False, _Fake(0x3002), stream=0)) == hk.EINVAL     # counter alignment
    assert code(lambda: hk.hikonv_epilogue(x, 1, 4, 8, 8, 40, 15, True, 4, hk.FMT_BITDENSE, y, stream=0)) == hk.EINVAL   # shift
    assert code(lambda: hk.hikonv_epilogue(x, 1, 4, 8, 8, 3, 16, True, 4, hk.FMT_BITDENSE, y, stream=0)) == hk.EINVAL    # qmax > 2^bits-1
    assert code(lambda: hk.hikonv_epilogue(x, 1, 4, 1, 8, 3, 15, True, 4, hk.FMT_BITDENSE, y, stream=0)) == hk.EINVAL    # nothing left after pooling
    assert code(lambda: hk.hikonv_ubench(99, 1, 1, _Fake(0x1000), stream=0)) in (hk.EUNSUPPORTED, hk.EHIP)
    assert code(lambda: hk.hikonv_conv1d_unpacked(4, 9, 0, x, hk.FMT_INT8, 2, 100, g, 3, hk.OUT_FULL, y, stream=0)) == hk.EINVAL
