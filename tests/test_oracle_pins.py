"""Pins of the direct-definition oracle (oracle/hikonv_oracle.c) against things other than
itself: library routines on textbook special cases, brute-force loops, the paper's worked
example, and invariants.  CPU only."""
import numpy as np
import pytest
import torch

from conftest import read_golden
from oracle import direct

RNG = np.random.default_rng(1234)


def _rand(shape, bits, signed):
    lo, hi = (-(1 << (bits - 1)), (1 << (bits - 1)) - 1) if signed else (0, (1 << bits) - 1)
    return RNG.integers(lo, hi + 1, size=shape, dtype=np.int8 if signed else np.uint8)


@pytest.mark.parametrize("bits,signed", [(1, False), (1, True), (4, False), (4, True), (8, False), (8, True)])
@pytest.mark.parametrize("taps", [1, 2, 3, 5, 7])
def test_conv1d_matches_numpy_convolve(bits, signed, taps):
    for length in (1, 2, 3, 7, 64, 257):
        x = _rand((3, length), bits, signed)
        g = _rand((taps,), bits, signed)
        full = direct.conv1d(x, g, direct.FULL)
        valid = direct.conv1d(x, g, direct.VALID)
        for r in range(3):
            ref = np.convolve(x[r].astype(np.int64), g.astype(np.int64), "full")
            assert np.array_equal(full[r], ref)
            if length >= taps:
                assert np.array_equal(valid[r], np.convolve(x[r].astype(np.int64), g.astype(np.int64), "valid"))
            else:
                assert valid.shape[1] == 0


def test_conv1d_brute_force_tiny():
    # y[m] = sum over all (n, k) with n + k = m  (Eq. ym), written as a double loop.
    f = [3, -2, 5, 7, -8]
    g = [2, -1, 4]
    y = [0] * (len(f) + len(g) - 1)
    for n, fv in enumerate(f):
        for k, gv in enumerate(g):
            y[n + k] += fv * gv
    got = direct.conv1d(np.array(f, dtype=np.int8), np.array(g, dtype=np.int8), direct.FULL)
    assert got.tolist() == y
    got_v = direct.conv1d(np.array(f, dtype=np.int8), np.array(g, dtype=np.int8), direct.VALID)
    assert got_v.tolist() == y[len(g) - 1:len(f)]


def test_conv1d_worked_example_from_paper():
    gold = read_golden("worked_example_f32.txt")
    f = np.array([int(v) for v in gold["f"].split()], dtype=np.uint8)
    g = np.array([int(v) for v in gold["g"].split()], dtype=np.uint8)
    assert direct.conv1d(f, g, direct.FULL).tolist() == [int(v) for v in gold["y"].split()]


def test_conv1d_is_true_convolution_not_correlation():
    # an asymmetric kernel: delta at k=1 delays the input by one (a correlation would advance it)
    f = np.arange(1, 9, dtype=np.int8)
    g = np.array([0, 1, 0, 0], dtype=np.int8)
    y = direct.conv1d(f, g, direct.FULL)
    assert y.tolist() == [0] + list(range(1, 9)) + [0, 0]


def test_conv1d_linearity_and_shift():
    x1, x2 = _rand((2, 50), 4, True), _rand((2, 50), 4, True)
    g = _rand((5,), 4, True)
    s = (x1.astype(np.int16) + x2.astype(np.int16))
    assert np.abs(s).max() < 128
    lhs = direct.conv1d(s.astype(np.int8), g)
    assert np.array_equal(lhs, direct.conv1d(x1, g) + direct.conv1d(x2, g))
    shifted = np.concatenate([np.zeros((2, 3), np.int8), x1], axis=1)
    assert np.array_equal(direct.conv1d(shifted, g)[:, 3:], direct.conv1d(x1, g))


def test_conv1d_extreme_values_do_not_wrap():
    x = np.full((1, 4), -128, dtype=np.int8)
    g = np.full((3,), -128, dtype=np.int8)
    assert direct.conv1d(x, g).tolist() == [[16384, 32768, 49152, 49152, 32768, 16384]]
    xu = np.full((1, 4), 255, dtype=np.uint8)
    assert direct.conv1d(xu, g).tolist() == [[-32640, -65280, -97920, -97920, -65280, -32640]]


@pytest.mark.parametrize("stride,pad", [(1, 0), (1, 1), (2, 1), (1, 2), (2, 0)])
@pytest.mark.parametrize("signed", [(True, True), (False, True), (False, False)])
def test_conv2d_matches_torch(stride, pad, signed):
    a_s, w_s = signed
    x = _rand((2, 5, 9, 11), 4, a_s)
    w = _rand((4, 5, 3, 3), 4, w_s)
    got = direct.conv2d(x, w, stride, pad)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)),
                                     torch.from_numpy(w.astype(np.float64)), stride=stride, padding=pad)
    assert np.array_equal(got, ref.numpy().astype(np.int64))


def test_conv2d_rectangular_kernels_match_torch():
    for kh, kw in ((1, 1), (1, 3), (3, 1), (5, 5), (2, 4)):
        x = _rand((1, 3, 8, 10), 8, False)
        w = _rand((2, 3, kh, kw), 8, True)
        got = direct.conv2d(x, w, 1, 0)
        ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)),
                                         torch.from_numpy(w.astype(np.float64)))
        assert np.array_equal(got, ref.numpy().astype(np.int64))


def test_conv2d_brute_force_tiny():
    x = _rand((1, 2, 4, 5), 3, True)
    w = _rand((2, 2, 3, 2), 3, True)
    pad, stride = 1, 2
    n, c, h, wd = x.shape
    co, _, kh, kw = w.shape
    xp = np.zeros((n, c, h + 2 * pad, wd + 2 * pad), dtype=np.int64)
    xp[:, :, pad:pad + h, pad:pad + wd] = x
    ho, wo = (h + 2 * pad - kh) // stride + 1, (wd + 2 * pad - kw) // stride + 1
    ref = np.zeros((n, co, ho, wo), dtype=np.int64)
    for o in range(co):
        for i in range(ho):
            for j in range(wo):
                ref[0, o, i, j] = int((xp[0, :, i * stride:i * stride + kh, j * stride:j * stride + kw]
                                       * w[o].astype(np.int64)).sum())
    assert np.array_equal(direct.conv2d(x, w, stride, pad), ref)


def test_conv2d_is_cross_correlation():
    # a kernel that is 1 at (kh, kw) = (0, 2) reads the pixel two to the right, same row
    x = np.arange(1, 31, dtype=np.int8).reshape(1, 1, 5, 6)
    w = np.zeros((1, 1, 3, 3), dtype=np.int8)
    w[0, 0, 0, 2] = 1
    y = direct.conv2d(x, w, 1, 0)
    assert np.array_equal(y[0, 0], x[0, 0, 0:3, 2:6])


@pytest.mark.parametrize("stride,pad", [(1, 0), (1, 1), (2, 1), (2, 0), (3, 2)])
@pytest.mark.parametrize("signed", [(True, True), (False, True), (False, False)])
def test_conv3d_matches_torch(stride, pad, signed):
    a_s, w_s = signed
    x = _rand((2, 3, 6, 7, 9), 4, a_s)
    w = _rand((4, 3, 3, 2, 3), 4, w_s)
    got = direct.conv3d(x, w, stride, pad)
    ref = torch.nn.functional.conv3d(torch.from_numpy(x.astype(np.float64)),
                                     torch.from_numpy(w.astype(np.float64)), stride=stride, padding=pad)
    assert np.array_equal(got, ref.numpy().astype(np.int64))


def test_conv3d_brute_force_tiny():
    x = _rand((1, 2, 3, 4, 5), 3, True)
    w = _rand((2, 2, 2, 3, 2), 3, True)
    pad, stride = 1, 2
    n, c, d, h, wd = x.shape
    co, _, kd, kh, kw = w.shape
    xp = np.zeros((n, c, d + 2 * pad, h + 2 * pad, wd + 2 * pad), dtype=np.int64)
    xp[:, :, pad:pad + d, pad:pad + h, pad:pad + wd] = x
    do, ho, wo = ((d + 2 * pad - kd) // stride + 1, (h + 2 * pad - kh) // stride + 1,
                  (wd + 2 * pad - kw) // stride + 1)
    ref = np.zeros((n, co, do, ho, wo), dtype=np.int64)
    for o in range(co):
        for a in range(do):
            for i in range(ho):
                for j in range(wo):
                    ref[0, o, a, i, j] = int((xp[0, :, a * stride:a * stride + kd, i * stride:i * stride + kh,
                                                 j * stride:j * stride + kw] * w[o].astype(np.int64)).sum())
    assert np.array_equal(direct.conv3d(x, w, stride, pad), ref)


def test_conv3d_special_cases():
    # depth 1 with a depth-1 kernel is the 2-D layer; a kernel that is 1 at one position
    # (kd, kh, kw) = (1, 0, 2) reads that voxel (cross-correlation, no flip on any axis)
    x = _rand((2, 3, 1, 6, 7), 4, True)
    w = _rand((4, 3, 1, 3, 3), 4, True)
    assert np.array_equal(direct.conv3d(x, w, 1, 1 * 0)[:, :, 0], direct.conv2d(x[:, :, 0], w[:, :, 0], 1, 0))
    v = np.arange(1, 121, dtype=np.int8).reshape(1, 1, 4, 5, 6)
    k = np.zeros((1, 1, 2, 3, 3), dtype=np.int8)
    k[0, 0, 1, 0, 2] = 1
    assert np.array_equal(direct.conv3d(v, k, 1, 0)[0, 0], v[0, 0, 1:4, 0:3, 2:6])
    # linear in the kernel's depth slices: the 3-D layer is the sum over kd of 2-D layers on shifted depth slices
    x = _rand((1, 2, 4, 5, 6), 4, False)
    w = _rand((3, 2, 3, 3, 3), 4, True)
    y = direct.conv3d(x, w, 1, 0)
    for d in range(y.shape[2]):
        acc = sum(direct.conv2d(x[:, :, d + kd], w[:, :, kd], 1, 0).astype(np.int64) for kd in range(3))
        assert np.array_equal(y[:, :, d], acc)


def test_relu_requant_hand_values():
    acc = np.array([-5, 0, 1, 7, 8, 15, 16, 127, 128, 1000, -2**31, 2**31 - 1], dtype=np.int32)
    got = direct.relu_requant(acc, 3, 15)
    assert got.tolist() == [0, 0, 0, 0, 1, 1, 2, 15, 15, 15, 0, 15]
    assert direct.relu_requant(acc[:6], 0, 15).tolist() == [0, 0, 1, 7, 8, 15]


def test_maxpool_matches_torch():
    x = _rand((2, 3, 7, 10), 4, False).view(np.int8)
    got = direct.maxpool2x2(x)
    ref = torch.nn.functional.max_pool2d(torch.from_numpy(x.astype(np.float32)), 2).numpy()
    assert np.array_equal(got, ref.astype(np.int8))


def test_maxpool_commutes_with_monotone_requant():
    acc = RNG.integers(-500, 500, size=(1, 2, 6, 8), dtype=np.int32)
    a = direct.maxpool2x2(direct.relu_requant(acc, 4, 15))
    pooled = acc.reshape(1, 2, 3, 2, 4, 2).max(axis=(3, 5)).astype(np.int32)
    assert np.array_equal(a, direct.relu_requant(pooled, 4, 15))


def test_bitdense_layout():
    # 1-bit: the container stream is numpy's little-endian bit packing
    v = _rand((3, 70), 1, False)
    got = direct.bitdense_pack(v, 1)
    assert got.shape == (3, 12)
    ref = np.packbits(v, axis=1, bitorder="little")
    assert np.array_equal(got[:, :ref.shape[1]], ref) and not got[:, ref.shape[1]:].any()
    # 4-bit signed: two's-complement nibbles, element 0 in the low nibble
    v = np.array([[-8, 7, -1, 3, 5]], dtype=np.int8)
    got = direct.bitdense_pack(v, 4)
    assert got.tolist() == [[0x78, 0x3F, 0x05, 0x00]]
    # 3-bit values sit in 4-bit containers with the top container bit clear
    v = np.array([[-4, 3, -1]], dtype=np.int8)
    assert direct.bitdense_pack(v, 3).tolist() == [[0x34, 0x07, 0, 0]]
    # 2-bit: four per byte; 5..8-bit: one per byte, masked to b bits
    assert direct.bitdense_pack(np.array([[1, 2, 3, 0, -1]], dtype=np.int8), 2).tolist() == [[0x39, 0x03, 0, 0]]
    assert direct.bitdense_pack(np.array([[-1, 5]], dtype=np.int8), 6).tolist() == [[0x3F, 5, 0, 0]]
    assert direct.bitdense_row_bytes(65536, 4) == 32768 and direct.bitdense_row_bytes(9, 1) == 4
