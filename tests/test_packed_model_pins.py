"""Pins of the big-integer packed model (oracle/packed_model.py): the values the paper prints
for its worked example, the multi-channel identity it builds on, and equality with the direct
definitions (library routines / brute force) on random, extreme and exhaustive inputs."""
import itertools

import numpy as np
import pytest

from conftest import read_golden
from oracle import direct, packed_model as pm, plan_model as pl

RNG = np.random.default_rng(99)


def _range(bits, signed):
    return (-(1 << (bits - 1)), (1 << (bits - 1)) - 1) if signed else (0, (1 << bits) - 1)


def _rand(n, bits, signed):
    lo, hi = _range(bits, signed)
    return [int(v) for v in RNG.integers(lo, hi + 1, size=n)]


def test_worked_example_integers():
    gold = read_golden("worked_example_f32.txt")
    f = [int(v) for v in gold["f"].split()]
    g = [int(v) for v in gold["g"].split()]
    s = int(gold["slice_bits"])
    # the figure stores element 0 in the top slice: pack the reversed sequences
    a, b = pm.pack(f[::-1], s), pm.pack(g[::-1], s)
    assert a == int(gold["multiplicand_a"]) and b == int(gold["multiplicand_b"])
    assert a * b == int(gold["product"]) == int(gold["product_binary"], 2)
    segs = pm.split_unsigned(a * b, s, len(f) + len(g) - 1)
    assert segs[::-1] == [int(v) for v in gold["y"].split()]
    # Eq. (inpack) order (element 0 in the low slice) gives the same outputs, low segment first
    y, _ = pm.fnk(f, g, s, False)
    assert y == [int(v) for v in gold["y"].split()]


def test_multichannel_int4_identity():
    # Eq. (xilinx4bit): (V2*2^11 + V1)(W2*2^22 + W1), V unsigned 4-bit, W signed 4-bit,
    # gives V1W1, V2W1, V1W2, V2W2 at bit offsets 0, 11, 22, 33.
    for v1, v2 in itertools.product(range(16), repeat=2):
        for w1, w2 in itertools.product(range(-8, 8), repeat=2):
            prod = (v2 * 2 ** 11 + v1) * (w2 * 2 ** 22 + w1)
            assert prod == pm.pack([v1, v2], 11) * pm.pack([w1, 0, w2], 11)
            assert pm.split_signed(prod, 11, 4) == [v1 * w1, v2 * w1, v1 * w2, v2 * w2]
            assert pm.split_signed_bias(prod, 11, 4) == [v1 * w1, v2 * w1, v1 * w2, v2 * w2]


@pytest.mark.parametrize("bits", range(1, 9))
@pytest.mark.parametrize("signs", [(False, False), (True, True), (False, True), (True, False)])
def test_theorem1_polynomial_identity(bits, signs):
    plan = pl.paper_search(bits, bits, 32, 32, pl.SINGLE)
    n, k, s = plan["N"], plan["K"], plan["S"]
    if bits == 1 and any(signs):
        s += 1            # signed 1-bit values {-1,0}: the printed slice is one bit short (see plan tests)
    cases = [(_rand(n, bits, signs[0]), _rand(k, bits, signs[1])) for _ in range(50)]
    for fa, ga in itertools.product(_range(bits, signs[0]), _range(bits, signs[1])):
        cases.append(([fa] * n, [ga] * k))
    for f, g in cases:
        y_ref = np.convolve(np.array(f, dtype=np.int64), np.array(g, dtype=np.int64)).tolist()
        prod = pm.pack(f, s) * pm.pack(g, s)
        assert prod == sum(v << (s * m) for m, v in enumerate(y_ref))          # Eq. (prod)
        y, _ = pm.fnk(f, g, s, any(signs))
        assert y == y_ref


def test_signed_slice_packing_equals_shift_add():
    for bits, s, n in ((4, 10, 3), (2, 6, 5), (8, 18, 2), (1, 4, 8), (3, 8, 4)):
        for _ in range(200):
            f = _rand(n, bits, True)
            assert pm.pack_slices_signed(f, s) == pm.pack(f, s) % (1 << (s * n))


def test_signed_split_exhaustive_small():
    for bits in (1, 2):
        lo, hi = _range(bits, True)
        vals = range(lo, hi + 1)
        for n, k in itertools.product((1, 2, 3), repeat=2):
            s = pl.slice_bits(bits, bits, pl.guard_bits(pl.SINGLE, n, k)) + (1 if bits == 1 else 0)
            for f in itertools.product(vals, repeat=n):
                for g in itertools.product(vals, repeat=k):
                    ref = np.convolve(np.array(f, dtype=np.int64), np.array(g, dtype=np.int64)).tolist()
                    prod = pm.pack(f, s) * pm.pack(g, s)
                    assert pm.split_signed(prod, s, n + k - 1) == ref
                    assert pm.split_signed_bias(prod, s, n + k - 1) == ref


@pytest.mark.parametrize("bits", range(1, 9))
@pytest.mark.parametrize("signs", [(False, False), (True, True), (False, True)])
@pytest.mark.parametrize("taps", [3, 5, 7])
def test_theorem2_overlap_add_equals_direct(bits, signs, taps):
    plan = pl.paper_search_taps(bits, bits, 32, 32, taps, pl.CONV1D)
    n, k, s = plan["N"], plan["K"], plan["S"]
    if bits == 1 and any(signs):
        s += 1
    lo_f, hi_f = _range(bits, signs[0])
    for length in (1, n - 1 or 1, n, n + 1, 3 * n + 2, 50):
        inputs = [_rand(length, bits, signs[0]), [lo_f] * length, [hi_f] * length]
        for f in inputs:
            for g in (_rand(taps, bits, signs[1]), [_range(bits, signs[1])[0]] * taps,
                      [_range(bits, signs[1])[1]] * taps):
                fa = np.array(f, dtype=np.int8 if signs[0] else np.uint8)
                ga = np.array(g, dtype=np.int8 if signs[1] else np.uint8)
                ref = direct.conv1d(fa, ga, direct.FULL).tolist()
                assert pm.conv1d_packed(f, g, n, k, s, any(signs)) == ref


def test_guard_bits_are_sufficient_and_tight():
    # unsigned 4-bit, three products per segment: 3*15*15 = 675 needs 10 bits
    f, g = [15] * 3, [15] * 3
    ref = np.convolve(f, g).tolist()
    assert max(ref) == 675
    assert pm.fnk(f, g, 10, False)[0] == ref                      # G_b = 2: exact
    assert pm.fnk(f, g, 9, False)[0] != ref                       # G_b = 1: fields collide
    # 1-D mode with K=3 and a long row: still exact at S=10
    assert pm.conv1d_packed([15] * 20, g, 3, 3, 10, False) == np.convolve([15] * 20, g).tolist()
    assert pm.conv1d_packed([15] * 20, g, 3, 3, 9, False) != np.convolve([15] * 20, g).tolist()


def test_signed_one_bit_needs_one_more_slice_bit():
    # values {-1,0}: (-1)*(-1) = +1, eight of them sum to 8 = 2^(S-1) for the printed S=4
    f, g = [-1] * 8, [-1] * 8
    ref = np.convolve(f, g).tolist()
    assert pm.fnk(f, g, 4, True)[0] != ref
    assert pm.fnk(f, g, 5, True)[0] == ref


@pytest.mark.parametrize("signs", [(False, False), (True, True), (False, True)])
def test_theorem3_dnn_mapping_with_accumulation(signs):
    bits = 4
    rng = np.random.default_rng(5)
    lo_a, hi_a = _range(bits, signs[0])
    lo_w, hi_w = _range(bits, signs[1])
    for (c, h, w, co, kh, kw, pad, m_acc) in [(3, 5, 7, 2, 3, 3, 1, 5), (4, 4, 9, 3, 3, 3, 0, 4),
                                              (2, 6, 6, 2, 1, 1, 0, 2), (5, 3, 8, 2, 3, 5, 2, 3)]:
        gb = pl.ceil_log2(m_acc * kw)
        s = pl.slice_bits(bits, bits, gb)
        n, k = 3, min(kw, 3)
        x = rng.integers(lo_a, hi_a + 1, size=(1, c, h, w), dtype=np.int8 if signs[0] else np.uint8)
        wt = rng.integers(lo_w, hi_w + 1, size=(co, c, kh, kw), dtype=np.int8 if signs[1] else np.uint8)
        for xv, wv in ((x, wt), (np.full_like(x, lo_a if signs[0] else hi_a), np.full_like(wt, lo_w if signs[1] else hi_w))):
            ref = direct.conv2d(xv, wv, 1, pad)[0]
            got = pm.conv2d_packed(xv[0].tolist(), wv.tolist(), pad, n, k, s, m_acc, any(signs))
            assert np.array_equal(np.array(got), ref)


def test_overlap_add_with_kernel_longer_than_block():
    # K-1 > N: a block product reaches past its neighbour; the stored word carries it on
    for n, k, s in ((1, 3, 10), (2, 5, 11), (1, 4, 10), (2, 4, 10)):
        for _ in range(20):
            f, g = _rand(17, 4, False), _rand(k, 4, False)
            assert pm.conv1d_packed(f, g, n, k, s, False) == np.convolve(f, g).tolist()
        f, g = _rand(17, 3, True), _rand(k, 3, True)
        assert pm.conv1d_packed(f, g, n, k, s, True) == np.convolve(f, g).tolist()


def test_bipolar_values_as_signed_slices():
    # {-1,+1} data with zero padding are three-valued; as signed slices the products are -1, 0, 1,
    # so a 10-bit slice holds 170 accumulated (channel, kernel-row) products of 3 taps (|sum| <= 510)
    # and four such slices fill a signed 32-bit word.  One more product per segment does not fit.
    s, n, k = 10, 4, 3
    assert abs(pm.pack([-1] * n, s)) < 2 ** 31 and pm.pack([1] * n, s) < 2 ** 31
    assert abs(pm.pack([-1] * (n + 1), s)) >= 2 ** 31           # a fifth slice overflows the signed word
    rng = np.random.default_rng(11)
    x = (rng.integers(0, 2, size=(1, 6, 5, 9)) * 2 - 1).astype(np.int8)
    wt = (rng.integers(0, 2, size=(3, 6, 3, 3)) * 2 - 1).astype(np.int8)
    ref = direct.conv2d(x, wt, 1, 1)[0]
    assert np.array_equal(np.array(pm.conv2d_packed(x[0].tolist(), wt.tolist(), 1, n, k, s, 170, True)), ref)
    # every segment at its bound: 170 x 3 products of (+1)(-1) or (-1)(-1)
    for av, wv in itertools.product((-1, 1), (-1, 1)):
        xe = np.full((1, 170, 1, 12), av, dtype=np.int8)
        we = np.full((1, 170, 1, 3), wv, dtype=np.int8)
        ref = direct.conv2d(xe, we, 1, 1)[0]
        assert np.array_equal(np.array(pm.conv2d_packed(xe[0].tolist(), we.tolist(), 1, n, k, s, 170, True)), ref)
    xe = np.full((1, 171, 1, 12), 1, dtype=np.int8)
    we = np.full((1, 171, 1, 3), -1, dtype=np.int8)
    bad = pm.conv2d_packed(xe[0].tolist(), we.tolist(), 1, n, k, s, 171, True)
    assert not np.array_equal(np.array(bad), direct.conv2d(xe, we, 1, 1)[0])     # -513 leaves the 10-bit field


@pytest.mark.parametrize("stride,kw,pad", [(2, 3, 1), (2, 5, 2), (3, 5, 1), (2, 7, 3), (4, 4, 0), (2, 3, 4)])
def test_polyphase_identity_of_a_strided_layer(stride, kw, pad):
    # O[w] = sum_p sum_j Ipad_p[w+j] W[j*s+p] with Ipad_p[i] = Ipad[s*i+p]: a stride-s row convolution is the
    # sum over the s column phases of stride-1 convolutions with the phase kernels (zero beyond Kw); checked
    # with the direct definitions only (columns of the layer), then through the packed model
    rng = np.random.default_rng(stride * 100 + kw)
    c, h, w, co, kh = 3, 6, 19, 2, 3
    x = rng.integers(-8, 8, size=(1, c, h, w), dtype=np.int8)
    wt = rng.integers(-8, 8, size=(co, c, kh, kw), dtype=np.int8)
    ref = direct.conv2d(x, wt, stride, pad)
    wo = ref.shape[3]
    kp = -(-kw // stride)
    # phase tensors: channel (ci, p) holds the padded row at s*i + p; kernel (ci, p) holds taps j*s + p
    xp = np.zeros((1, c, h, w + 2 * pad + stride * kp), dtype=np.int8)
    xp[:, :, :, pad:pad + w] = x
    xph = np.zeros((1, c * stride, h, wo + kp - 1), dtype=np.int8)
    wph = np.zeros((co, c * stride, kh, kp), dtype=np.int8)
    for ci in range(c):
        for p in range(stride):
            xph[0, ci * stride + p] = xp[0, ci, :, p::stride][:, :wo + kp - 1]
            taps = wt[:, ci, :, p::stride]
            wph[:, ci * stride + p, :, :taps.shape[2]] = taps
    # rows still step by `stride` and keep their vertical padding: take every stride-th row of a stride-1 layer
    xv = np.zeros((1, c * stride, h + 2 * pad, wo + kp - 1), dtype=np.int8)
    xv[:, :, pad:pad + h] = xph
    got = direct.conv2d(xv, wph, 1, 0)[:, :, ::stride][:, :, :ref.shape[2]]
    assert np.array_equal(got, ref)
    packed = pm.conv2d_packed(xv[0].tolist(), wph.tolist(), 0, 3, min(kp, 3), 16, 4, True)
    assert np.array_equal(np.array(packed)[:, ::stride][:, :ref.shape[2]], ref[0])


def test_volume_layer_is_an_outer_sum_over_kernel_depth():
    # every (channel, kernel depth slice) pair of a 3-D layer is a channel of a 2-D layer on the input's depth
    # slice d + kd: the packed model run on those stacked channels equals the direct 3-D definition
    rng = np.random.default_rng(21)
    c, d, h, w, co, kd, kh, kw = 2, 4, 5, 8, 2, 3, 3, 3
    x = rng.integers(-8, 8, size=(1, c, d, h, w), dtype=np.int8)
    wt = rng.integers(-8, 8, size=(co, c, kd, kh, kw), dtype=np.int8)
    ref = direct.conv3d(x, wt, 1, 0)
    for dd in range(ref.shape[2]):
        xs = np.concatenate([x[0, :, dd + k] for k in range(kd)], axis=0)             # [(kd, ci)][h][w]
        ws = np.concatenate([wt[:, :, k] for k in range(kd)], axis=1)                 # [co][(kd, ci)][kh][kw]
        got = pm.conv2d_packed(xs.tolist(), ws.tolist(), 0, 3, 3, 14, 6, True)
        assert np.array_equal(np.array(got), ref[0, :, dd])


@pytest.mark.parametrize("c,bits,signs,taps", [(4, 4, (False, False), 3), (4, 4, (True, True), 3), (4, 3, (False, True), 5),
                                               (1, 1, (False, False), 7), (2, 2, (True, False), 3), (8, 6, (True, True), 2)])
def test_container_aligned_slices_with_one_tap_per_word(c, bits, signs, taps):
    """Theorem 1 with K = 1 and the elements dealt to the slices J = 16/c apart: the word for residue
    rho holds elements rho and rho + J of a window in two 16-bit slices, a tap multiplies it as a
    plain integer, the taps accumulate in the packed domain, and the two slices of the sum are
    outputs rho and rho + J.  In exact integers, against the direct definition."""
    a_s, w_s = signs
    j, per = 16 // c, 32 // c
    f, g = _rand(5 * per + taps - 1, bits, a_s), _rand(taps, bits, w_s)
    ref = direct.conv1d(np.array([f]), np.array(g), direct.VALID)[0]
    any_signed = a_s or w_s
    got = []
    for k in range(5):                                   # output dword k: outputs k*per .. k*per + per - 1
        win = f[k * per:k * per + per + taps - 1]        # window element t = f[k*per + t]
        out = [None] * per
        for rho in range(j):
            y = 0
            for kk in range(taps):
                tau = rho + taps - 1 - kk
                y += pm.pack([win[tau], win[tau + j]], 16) * g[kk]
            fields = pm.split_signed_bias(y, 16, 2) if any_signed else pm.split_unsigned(y, 16, 2)
            out[rho], out[rho + j] = fields
        got += out
    assert got == [int(v) for v in ref[:5 * per]]


def test_container_aligned_slices_need_the_sum_to_fit_sixteen_bits():
    # 8-bit unsigned, 3 taps: 3 * 255 * 255 does not fit 16 bits and the low slice spills into the high one
    f, g = [255] * 6, [255] * 3
    y = sum(pm.pack([f[t], f[t + 2]], 16) * g[k] for k, t in enumerate((2, 1, 0)))
    assert pm.split_unsigned(y, 16, 2) != [3 * 255 * 255] * 2
    # one tap fits: 255 * 255 < 2**16
    assert pm.split_unsigned(pm.pack([255, 255], 16) * 255, 16, 2) == [255 * 255] * 2
    # signed 7-bit, 2 taps: |sum| <= 2 * 64 * 64 = 2**13 fits the signed slice; the library's bound is |sum| < 2**15
    y = pm.pack([-64, -64], 16) * -64 + pm.pack([-64, -64], 16) * -64
    assert pm.split_signed_bias(y, 16, 2) == [8192, 8192]
