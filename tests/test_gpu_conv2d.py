"""GPU parity: packed DNN layer (wide and 24-bit multipliers, {-1,+1} layers), unpacked
baseline, epilogue and the chained CNN, through the C ABI vs the int64 oracle, bit-exact."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import direct

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_00763_amd as hk
    from paper_2208_00763_amd.cnn import PackedCnn, UnpackedCnn
    from gpu_util import run_conv2d, dnn_plan, dev, compact, Guarded, oracle_cnn

SHAPES = [  # n, c, h, w, co, kh, kw, stride, pad
    (1, 3, 5, 7, 2, 3, 3, 1, 1),
    (2, 5, 9, 11, 9, 3, 3, 1, 0),
    (1, 4, 8, 8, 16, 1, 1, 1, 0),
    (1, 6, 10, 13, 4, 3, 3, 2, 1),
    (1, 2, 7, 20, 3, 5, 5, 1, 2),
    (1, 7, 6, 9, 10, 3, 2, 1, 1),
    (1, 3, 4, 70, 2, 3, 3, 1, 1),
]


def _case(bits, a_s, w_s, shape, tag):
    n, c, h, w, co, kh, kw, _, _ = shape
    rng = wl.rng_for(tag, bits, a_s, w_s, shape)
    return wl.uniform_values(rng, (n, c, h, w), bits, a_s), wl.uniform_values(rng, (co, c, kh, kw), bits, w_s)


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 6, 8])
@pytest.mark.parametrize("signs", [(False, False), (True, True), (False, True)])
def test_conv2d_packed_small_shapes(bits, signs):
    a_s, w_s = signs
    ran = 0
    for shape in SHAPES:
        x, w = _case(bits, a_s, w_s, shape, "d1")
        stride, pad, kw = shape[7], shape[8], shape[6]
        ref = direct.conv2d(x, w, stride, pad)
        for wide in (True, False):
            for m in (1, 4, 0):
                try:
                    plan = dnn_plan(bits, bits, a_s, w_s, kw, m, wide)
                except hk.HikonvError as e:
                    assert e.code == hk.ENOPLAN
                    continue
                for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
                    got = run_conv2d(plan, x, w, stride, pad, fmt, prepacked=(m == 4))
                    assert np.array_equal(got, ref), (bits, signs, shape, wide, m, fmt, plan)
                    ran += 1
    assert ran > 0


@pytest.mark.parametrize("wide", [True, False])
def test_conv2d_long_rows_are_segmented(wide):
    # rows of more than 63 packed blocks are cut into wave segments with a recomputed halo block
    for bits, a_s, w_s, width in ((4, True, True, 400), (1, False, False, 1200), (2, False, True, 333)):
        shape = (1, 3, 3, width, 4, 3, 3, 1, 1)
        x, w = _case(bits, a_s, w_s, shape, "d2")
        try:
            plan = dnn_plan(bits, bits, a_s, w_s, 3, 3, wide)
        except hk.HikonvError as e:
            assert e.code == hk.ENOPLAN    # no plan exists for this request; nothing is skipped silently
            continue
        assert (width + 1 + plan.N - 1) // plan.N > 63
        assert np.array_equal(run_conv2d(plan, x, w, 1, 1), direct.conv2d(x, w, 1, 1))


def test_conv2d_extreme_values():
    for bits, a_s, w_s in ((4, True, True), (4, False, True), (4, False, False), (2, True, True), (8, True, True)):
        lo_a, hi_a = wl.value_range(bits, a_s)
        lo_w, hi_w = wl.value_range(bits, w_s)
        for av in (lo_a, hi_a):
            for wv in (lo_w, hi_w):
                x = np.full((1, 20, 6, 9), av, dtype=np.int8 if a_s else np.uint8)
                w = np.full((3, 20, 3, 3), wv, dtype=np.int8 if w_s else np.uint8)
                plan = dnn_plan(bits, bits, a_s, w_s, 3, 0, True)
                assert np.array_equal(run_conv2d(plan, x, w, 1, 1), direct.conv2d(x, w, 1, 1)), (bits, av, wv, plan)


def test_conv2d_config3_full():
    x, w = wl.config3()
    ref = direct.conv2d(x, w, 1, 1)
    for m in (5, 0):
        plan = dnn_plan(4, 4, True, True, 3, m, True)
        assert np.array_equal(run_conv2d(plan, x, w, 1, 1, hk.FMT_BITDENSE, prepacked=True), ref)
    plan = dnn_plan(4, 4, True, True, 3, 5, True)
    assert (plan.N, plan.K, plan.S) == (3, 3, 12)


@pytest.mark.parametrize("shape", [(1, 4, 6, 7, 5, 3, 3, 1, 1), (2, 16, 9, 9, 9, 3, 3, 1, 0), (1, 8, 8, 10, 4, 3, 3, 2, 1),
                                   (1, 5, 5, 5, 3, 1, 1, 1, 0), (1, 33, 7, 30, 8, 3, 3, 1, 1)])
def test_conv2d_bipolar_small(shape):
    n, c, h, w, co, kh, kw, stride, pad = shape
    x, wt = wl.bipolar_case(n, c, h, w, co, kh, kw, tag="d3")
    ref = direct.conv2d(x, wt, stride, pad)
    for wide in (True, False):
        for m in (3, 0):
            plan = dnn_plan(1, 1, False, False, kw, m, wide, bipolar=True)
            for fmt in (hk.FMT_INT8, hk.FMT_BITDENSE):
                got = run_conv2d(plan, x, wt, stride, pad, fmt, prepacked=(m == 3))
                assert np.array_equal(got, ref), (shape, wide, m, fmt, plan)


def test_conv2d_config4_full():
    x, w = wl.config4()
    assert x.shape == (8, 256, 28, 28) and w.shape == (256, 256, 3, 3)
    ref = direct.conv2d(x, w, 1, 1)
    for wide in (True, False):
        plan = dnn_plan(1, 1, False, False, 3, 0, wide, bipolar=True)
        assert plan.N <= hk.LAYER_MAX_N
        assert np.array_equal(run_conv2d(plan, x, w, 1, 1, hk.FMT_BITDENSE, prepacked=True), ref)


def test_conv2d_unpacked_baseline():
    for bits, a_s, w_s in ((4, True, True), (8, False, True), (1, False, False)):
        for shape in SHAPES:
            x, w = _case(bits, a_s, w_s, shape, "d4")
            n, c, h, wd, co, kh, kw, stride, pad = shape
            ho, wo = (h + 2 * pad - kh) // stride + 1, (wd + 2 * pad - kw) // stride + 1
            y = torch.zeros(n * co * ho * wo, dtype=torch.int32, device="cuda")
            hk.hikonv_conv2d_unpacked(bits, bits, hk.signedness(a_s, w_s), dev(x), n, c, h, wd, dev(w), co, kh, kw,
                                      stride, pad, y)
            torch.cuda.synchronize()
            assert np.array_equal(y.cpu().numpy().reshape(n, co, ho, wo), direct.conv2d(x, w, stride, pad))
    x, w = wl.config4(8)
    n, c, h, wd = x.shape
    co = w.shape[0]
    y = torch.zeros(n * co * h * wd, dtype=torch.int32, device="cuda")
    hk.hikonv_conv2d_unpacked(1, 1, hk.BIPOLAR, dev(x), n, c, h, wd, dev(w), co, 3, 3, 1, 1, y)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().reshape(n, co, h, wd), direct.conv2d(x, w, 1, 1))


def test_compact_matches_oracle_layout():
    # row lengths that are and are not multiples of 4 (the streaming kernel takes the first kind),
    # of 16 and of 32; rows ending inside a thread's group of values; one row longer than a workgroup's reach
    for bits in range(1, 9):
        for signed in (False, True):
            for rows, length in ((5, 1003), (3, 4), (7, 16), (4, 20), (3, 36), (5, 1000), (2, 1028), (3, 8192 + 44),
                                 (70000, 12)):
                x = wl.uniform_values(wl.rng_for("cp", bits, signed, length), (rows, length), bits, signed)
                got = compact(x, bits).cpu().numpy()        # guard regions on both sides are checked inside
                ref = direct.bitdense_pack(x, bits)
                assert got.size == ref.size
                assert np.array_equal(got.reshape(ref.shape), ref), (bits, signed, rows, length)
    # {-1,+1} rows: bit 1 where the value is positive; any int8 value is a legal input byte
    for rows, length in ((3, 64), (5, 100), (2, 1003)):
        x = wl.bipolar_values(wl.rng_for("cpb", length), (rows, length))
        ref = direct.bitdense_pack(((x > 0).astype(np.int8)), 1)
        assert np.array_equal(compact(x, 1, bipolar=True).cpu().numpy().reshape(ref.shape), ref)
        odd = wl.rng_for("cpo", length).integers(-128, 128, (rows, length)).astype(np.int8)
        ref = direct.bitdense_pack(((odd > 0).astype(np.int8)), 1)
        assert np.array_equal(compact(odd, 1, bipolar=True).cpu().numpy().reshape(ref.shape), ref)


def test_check_range_counts_out_of_range_values():
    # counts are compared with a count in numpy over the same bytes; sizes below, at and above one grid stride
    rng = np.random.default_rng(11)
    for count in (1, 63, 64, 4097, 1 << 20, (8192 * 256) * 2 + 77):
        raw = rng.integers(-128, 128, count).astype(np.int8)
        x_d = dev(raw.view(np.uint8))
        for bits in range(1, 9):
            for signed in (False, True):
                v = raw.astype(np.int32) if signed else raw.view(np.uint8).astype(np.int32)
                lo, hi = (-(1 << (bits - 1)), (1 << (bits - 1)) - 1) if signed else (0, (1 << bits) - 1)
                n_bad = torch.full((1,), 5, dtype=torch.int32, device="cuda")      # the call adds to the counter
                hk.hikonv_check_range(x_d, count, bits, signed, False, n_bad)
                assert int(n_bad.item()) == 5 + int(((v < lo) | (v > hi)).sum()), (count, bits, signed)
        n_bad = torch.zeros(1, dtype=torch.int32, device="cuda")
        hk.hikonv_check_range(x_d, count, 1, False, True, n_bad)
        assert int(n_bad.item()) == int(((raw != 1) & (raw != -1)).sum())
    # in-range data of every kind the generators make: nothing counted
    for bits, signed in ((1, False), (4, True), (8, False), (8, True)):
        x = wl.uniform_values(wl.rng_for("rg", bits, signed), (7, 1001), bits, signed)
        n_bad = torch.zeros(1, dtype=torch.int32, device="cuda")
        hk.hikonv_check_range(dev(x), x.size, bits, signed, False, n_bad)
        assert int(n_bad.item()) == 0
    x = wl.bipolar_values(wl.rng_for("rgb"), (3, 999))
    n_bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    hk.hikonv_check_range(dev(x), x.size, 1, False, True, n_bad)
    assert int(n_bad.item()) == 0


def test_epilogue_matches_oracle():
    rng = np.random.default_rng(3)
    for (n, c, h, w, shift, pool) in ((1, 3, 6, 10, 3, True), (2, 5, 7, 9, 0, False), (1, 4, 9, 17, 5, True),
                                      (1, 2, 4, 64, 2, False), (1, 1, 2, 2100, 1, True), (1, 2, 3, 1031, 4, False),
                                      (2, 40000, 2, 2, 0, True), (1, 3, 5, 1, 0, False)):
        acc = rng.integers(-3000, 3000, size=(n, c, h, w), dtype=np.int32)
        q = direct.relu_requant(acc, shift, 15)
        if pool:
            q = direct.maxpool2x2(q)
        ho, wo = q.shape[2], q.shape[3]
        ref_bd = direct.bitdense_pack(q.reshape(n * c * ho, wo), 4)
        out_bd = Guarded(ref_bd.size, torch.uint8, 0xA5)
        hk.hikonv_epilogue(dev(acc), n, c, h, w, shift, 15, pool, 4, hk.FMT_BITDENSE, out_bd.view)
        out_i8 = Guarded(n * c * ho * wo, torch.uint8, 0xA5)
        hk.hikonv_epilogue(dev(acc), n, c, h, w, shift, 15, pool, 4, hk.FMT_INT8, out_i8.view)
        assert np.array_equal(out_bd.result().reshape(ref_bd.shape), ref_bd), (n, c, h, w, pool)
        assert np.array_equal(out_i8.result().reshape(q.shape), q.view(np.uint8)), (n, c, h, w, pool)


@pytest.mark.parametrize("pool", [0, 1])
@pytest.mark.parametrize("wide", [True, False])
def test_epilogue_pack_feeds_the_next_layer(pool, wide):
    """hikonv_epilogue_pack writes the next layer's packed words; that layer, called with
    FMT_PACKED, must give what the oracle gives for requantise -> pool -> convolution."""
    for (n, c, h, w, co, kh, kw, pad, shift, tight) in ((1, 5, 7, 9, 4, 3, 3, 1, 3, 0), (2, 16, 12, 30, 9, 3, 3, 1, 5, 1),
                                                        (1, 8, 9, 70, 8, 1, 1, 0, 0, 0), (1, 3, 10, 150, 5, 3, 5, 2, 4, 0),
                                                        (1, 4, 6, 8, 3, 5, 3, 0, 2, 0)):
        rng = wl.rng_for("epack", n, c, h, w, co, pool, wide)
        acc = rng.integers(-3000, 3000, size=(n, c, h, w)).astype(np.int32)
        wt = wl.uniform_values(rng, (co, c, kh, kw), 4, True)
        q = direct.relu_requant(acc, shift, 15)
        if pool:
            q = direct.maxpool2x2(q)
        hn, wn = q.shape[2], q.shape[3]
        if hn + 2 * pad < kh or wn + 2 * pad < kw:
            continue
        ref = direct.conv2d(q.view(np.uint8), wt, 1, pad)
        try:
            plan = dnn_plan(4, 4, False, True, kw, 0, wide, tight=tight)
        except hk.HikonvError as e:
            assert e.code == hk.ENOPLAN    # no plan exists for this request; nothing is skipped silently
            continue
        ws = torch.empty(hk.hikonv_conv2d_workspace_bytes(plan, n, c, hn, wn, co, kh, kw, 1, pad, True),
                         dtype=torch.uint8, device="cuda")
        pw = torch.empty(hk.hikonv_packed_weights_bytes(plan, co, c, kh, kw), dtype=torch.uint8, device="cuda")
        hk.hikonv_pack_weights(plan, dev(wt), co, c, kh, kw, pw)
        hk.hikonv_epilogue_pack(dev(acc), n, c, h, w, shift, 15, pool, plan, co, kh, kw, 1, pad, ws)
        y = torch.full((ref.size + 8,), -77777, dtype=torch.int32, device="cuda")
        hk.hikonv_conv2d_prepacked(plan, None, hk.FMT_PACKED, n, c, hn, wn, pw, co, kh, kw, 1, pad, ws, y)
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        assert (got[ref.size:] == -77777).all()
        assert np.array_equal(got[:ref.size].reshape(ref.shape), ref), (n, c, h, w, co, kh, kw, pad, pool, wide, plan)
    # argument checks: signed next-layer activations, qmax beyond the width, workspace too small
    plan = dnn_plan(4, 4, False, True, 3, 0, wide)
    acc_d = torch.zeros(64, dtype=torch.int32, device="cuda")
    ws = torch.empty(hk.hikonv_conv2d_workspace_bytes(plan, 1, 1, 8, 8, 2, 3, 3, 1, 1, True), dtype=torch.uint8,
                     device="cuda")
    for kwargs, code in ((dict(qmax=16), hk.EINVAL), (dict(shift=32), hk.EINVAL), (dict(ws=ws[:256]), hk.EWORKSPACE),
                         (dict(plan=dnn_plan(4, 4, True, True, 3, 0, wide)), hk.EUNSUPPORTED)):
        a = dict(qmax=15, shift=0, ws=ws, plan=plan)
        a.update(kwargs)
        with pytest.raises(hk.HikonvError) as e:
            hk.hikonv_epilogue_pack(acc_d, 1, 1, 8, 8, a["shift"], a["qmax"], 0, a["plan"], 2, 3, 3, 1, 1, a["ws"])
        assert e.value.code == code


@pytest.mark.parametrize("fused", ["layer", True, False])
@pytest.mark.parametrize("size", [(32, 64), (160, 320), (38, 70)])
def test_cnn_forward_config5(size, fused):
    h, w = size
    x, weights, specs = wl.config5(h, w)
    ref_accs, shifts = oracle_cnn(x, weights, specs)
    net = PackedCnn([dev(wt).view(torch.uint8).reshape(wt.shape) for wt in weights], specs, fused=fused,
                    tight=int(fused is True))
    x_bd = compact(x.reshape(3 * h, w), 4)
    _, accs = net.forward(x_bd, 1, h, w, shifts)
    torch.cuda.synchronize()
    for i, (got, ref) in enumerate(zip(accs, ref_accs)):
        assert np.array_equal(got.cpu().numpy().reshape(ref.shape), ref), "layer %d" % i
    if fused == "layer":
        assert all(net.layer_kernel), "every layer of this network fits the one-kernel-per-layer form"
        # the chain as the benchmark runs it: intermediate accumulators never stored
        # (the planner's cost objective, as there, and Algorithm 1's plans)
        for objective in (hk.OBJ_MEASURED_COST, hk.OBJ_PAPER_OPS):
            lean = PackedCnn([dev(wt).view(torch.uint8).reshape(wt.shape) for wt in weights], specs, fused="layer",
                             keep_accs=False, objective=objective)
            last, _ = lean.forward(x_bd, 1, h, w, shifts)
            torch.cuda.synchronize()
            assert all(lean.layer_kernel)
            assert np.array_equal(last.cpu().numpy().reshape(ref_accs[-1].shape), ref_accs[-1]), objective
    if fused is True:
        # the baseline chain (one multiply per product) that the benchmark times beside it
        base = UnpackedCnn([dev(wt).view(torch.uint8).reshape(wt.shape) for wt in weights], specs)
        _, accs_u = base.forward(dev(x), 1, h, w, shifts)
        torch.cuda.synchronize()
        for i, (got, ref) in enumerate(zip(accs_u, ref_accs)):
            assert np.array_equal(got.cpu().numpy().reshape(ref.shape), ref), "unpacked layer %d" % i
    # deep layers of a random-weight network go mostly to zero after ReLU, so every layer is
    # also checked in isolation on fresh uniform inputs of its own shape
    hh, ww = h, w
    for i, (wt, spec) in enumerate(zip(weights, specs)):
        co, c, kh, kw = wt.shape
        xi = wl.uniform_values(wl.rng_for("c5iso", i, h, w), (1, c, hh, ww), 4, False)
        plan = net.layers[i]["plan"]
        got = run_conv2d(plan, xi, wt, 1, spec["pad"], hk.FMT_BITDENSE, prepacked=True)
        assert np.array_equal(got, direct.conv2d(xi, wt, 1, spec["pad"])), "isolated layer %d" % i
        if spec["pool"]:
            hh, ww = hh // 2, ww // 2


def test_conv2d_degenerate_and_strided_shapes():
    cases = [  # n, c, h, w, co, kh, kw, stride, pad
        (2, 3, 1, 9, 4, 1, 3, 1, 1),      # one image row
        (1, 2, 9, 1, 3, 3, 1, 1, 0),      # one image column
        (3, 8, 11, 12, 17, 3, 3, 2, 1),   # batch, stride 2, channels not a multiple of 8
        (1, 1, 5, 5, 1, 3, 3, 1, 2),      # padding as wide as the kernel allows, single channels
        (1, 40, 6, 6, 8, 3, 3, 3, 0),     # stride 3
        (2, 9, 7, 130, 5, 3, 3, 1, 1),    # wide rows (several wave segments for short blocks)
    ]
    for shape in cases:
        stride, pad, kw = shape[7], shape[8], shape[6]
        for bits, a_s, w_s in ((4, False, True), (2, True, True), (1, False, False)):
            x, w = _case(bits, a_s, w_s, shape, "d5")
            ref = direct.conv2d(x, w, stride, pad)
            for m in (2, 0):
                plan = dnn_plan(bits, bits, a_s, w_s, kw, m, True)
                assert np.array_equal(run_conv2d(plan, x, w, stride, pad, hk.FMT_BITDENSE), ref), (shape, bits, m, plan)
        n, c, h, wd, co, kh, kw2 = shape[:7]
        xb, wb = wl.bipolar_case(n, c, h, wd, co, kh, kw2, tag="d5")
        plan = dnn_plan(1, 1, False, False, kw2, 0, True, bipolar=True)
        if plan.N <= 8:
            assert np.array_equal(run_conv2d(plan, xb, wb, stride, pad), direct.conv2d(xb, wb, stride, pad)), shape
