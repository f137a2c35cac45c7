"""Pins of the performance-model oracle (oracle/plan_model.py) against the numbers the
paper prints, and against a brute-force count of Eq. (tot_ops).  CPU only."""
import itertools

import pytest

from conftest import read_golden
from oracle import plan_model as pl

GOLD = read_golden("plan_values.txt")


@pytest.mark.parametrize("key", ["ops_27x18_1bit", "ops_27x18_4bit", "ops_27x18_8bit",
                                 "ops_32x32_4bit", "ops_32x32_8bit"])
def test_ops_per_multiply_printed_in_paper(key):
    _, dims, bits = key.split("_")
    l_a, l_b = (int(v) for v in dims.split("x"))
    b = int(bits[:-3])
    assert pl.paper_search(b, b, l_a, l_b, pl.SINGLE)["ops"] == int(GOLD[key])


def test_binary_27x18_configuration():
    r = pl.paper_search(1, 1, 27, 18, pl.SINGLE)
    n, k = (int(v) for v in GOLD["nk_27x18_1bit"].split())
    assert (r["N"], r["K"]) == (n, k)
    mul, add = (int(v) for v in GOLD["mul_add_27x18_1bit"].split())
    assert n * k == mul and (n - 1) * (k - 1) == add
    # the slice width printed with it (4) cannot hold nine slices in 27 bits; Eq. (slice1) gives 3
    assert r["S"] == 3 and 1 + (n - 1) * 4 > 27


def test_4bit_27x18_split_into_mults_and_adds():
    r = pl.paper_search(4, 4, 27, 18, pl.SINGLE)
    mul, add = (int(v) for v in GOLD["mul_add_27x18_4bit"].split())
    assert r["N"] * r["K"] == mul and (r["N"] - 1) * (r["K"] - 1) == add


def test_4bit_conv1d_plan_of_the_evaluation():
    n, k, gb, s = (int(v) for v in GOLD["conv1d_32x32_4bit"].split())
    r = pl.paper_search(4, 4, 32, 32, pl.CONV1D)
    assert (r["N"], r["K"], r["G_b"], r["S"]) == (n, k, gb, s)
    r3 = pl.paper_search_taps(4, 4, 32, 32, 3, pl.CONV1D)
    assert (r3["N"], r3["K"], r3["G_b"], r3["S"], r3["chunks"]) == (n, k, gb, s, 1)


def test_printed_128_binary_ops_is_not_reachable():
    printed = int(GOLD["ops_32x32_1bit_printed"])
    # (2N-1)(2K-1) = 2*ops-1 = 255: the only near-square factorisations are (8,9) and (9,8)
    pairs = [(n, k) for n in range(1, 33) for k in range(1, 33) if pl.ops_per_multiply(n, k) == printed]
    assert (9, 8) in pairs and (8, 9) in pairs
    for n, k in pairs:
        s = pl.slice_bits(1, 1, pl.guard_bits(pl.SINGLE, n, k))
        assert not pl.fits(1, 1, n, k, s, 32, 32)
    best = pl.paper_search(1, 1, 32, 32, pl.SINGLE)
    assert (best["N"], best["K"], best["S"], best["ops"]) == (8, 8, 4, 113)
    assert 2 * best["N"] * best["K"] == printed      # 128 = every MAC counted as two operations


def test_ops_formula_by_brute_force():
    # count the non-zero products and the additions of an N-by-K partial-convolution table
    for n, k in itertools.product(range(1, 9), repeat=2):
        terms = [0] * (n + k - 1)
        for i in range(n):
            for j in range(k):
                terms[i + j] += 1
        mults = sum(terms)
        adds = sum(t - 1 for t in terms)
        assert pl.ops_per_multiply(n, k) == mults + adds
        assert max(terms) == min(n, k)


def test_slice_rule_cases():
    assert pl.slice_bits(1, 5, 2) == 7 and pl.slice_bits(5, 1, 2) == 7 and pl.slice_bits(1, 1, 3) == 4
    assert pl.slice_bits(4, 4, 2) == 10 and pl.slice_bits(2, 3, 0) == 5
    assert [pl.ceil_log2(v) for v in (1, 2, 3, 4, 5, 8, 9)] == [0, 1, 2, 2, 3, 3, 4]


def test_regression_tables():
    # computed from Eq. (slice1)-(slice3); not printed in the paper (regression values)
    assert [pl.paper_search(b, b, 27, 18)["ops"] for b in range(1, 9)] == [60, 23, 11, 8, 8, 2, 2, 2]
    assert [pl.paper_search(b, b, 32, 32)["ops"] for b in range(1, 9)] == [113, 41, 25, 13, 13, 8, 5, 5]
    assert [pl.paper_search(b, b, 64, 64)["ops"] for b in range(1, 9)] == [313, 128, 85, 61, 41, 32, 25, 25]
    taps3 = [pl.paper_search_taps(b, b, 32, 32, 3) for b in range(1, 9)]
    assert [(r["N"], r["K"], r["S"], r["chunks"]) for r in taps3] == [
        (11, 3, 3, 1), (6, 3, 6, 1), (4, 3, 8, 1), (3, 3, 10, 1), (3, 3, 12, 1),
        (2, 2, 14, 2), (2, 2, 16, 2), (2, 2, 18, 2)]
