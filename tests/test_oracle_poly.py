"""Pins of the oracle's multilinear-extension routines (Section 3.3) against
brute force and closed forms (no GPU)."""
import random

from tests import pyref
from tests.pyref import R


def test_eq_is_equality_indicator_on_bits(orc):
    n = 4
    for x in range(1 << n):
        u = orc.to_bytes(pyref.bits_msb_first(x, n))
        tab = orc.to_ints(orc.eq_table(u, threads=2))
        assert tab == [1 if y == x else 0 for y in range(1 << n)]


def test_eq_table_matches_product_formula_and_sums_to_one(orc):
    rng = random.Random(21)
    for n in (0, 1, 3, 6):
        u = [rng.randrange(R) for _ in range(n)]
        tab = orc.to_ints(orc.eq_table(orc.to_bytes(u), threads=3)) if n else [1]
        assert tab == [pyref.eq(u, pyref.bits_msb_first(x, n)) for x in range(1 << n)]
        assert sum(tab) % R == 1


def test_eq_at_point(orc):
    rng = random.Random(22)
    u = [rng.randrange(R) for _ in range(7)]
    v = [rng.randrange(R) for _ in range(7)]
    assert orc.to_ints(orc.eq_at_point(orc.to_bytes(u), orc.to_bytes(v))) == [pyref.eq(u, v)]


def _mle_by_halving(arr, point):
    # independent route: bind the LAST coordinate (lowest bit) first
    cur = list(arr)
    for w in reversed(point):
        cur = [(cur[2 * i] + w * (cur[2 * i + 1] - cur[2 * i])) % R for i in range(len(cur) // 2)]
    return cur[0]


def test_mle_agrees_with_tensor_on_the_cube_and_with_halving(orc):
    rng = random.Random(23)
    n = 5
    arr = [rng.randrange(R) for _ in range(1 << n)]
    A = orc.to_bytes(arr)
    for x in (0, 1, 7, 18, 31):
        assert orc.to_ints(orc.mle_eval(A, orc.to_bytes(pyref.bits_msb_first(x, n)))) == [arr[x]]
    for _ in range(5):
        p = [rng.randrange(R) for _ in range(n)]
        got = orc.to_ints(orc.mle_eval(A, orc.to_bytes(p), threads=3))
        assert got == [pyref.mle(arr, p)] == [_mle_by_halving(arr, p)]


def test_index_convention_first_coordinate_is_top_bit(orc):
    # S = indicator of index 2 = (1,0) in two variables: S~(w0, w1) = w0 (1 - w1)
    S = orc.to_bytes([0, 0, 1, 0])
    w0, w1 = 5, 11
    assert orc.to_ints(orc.mle_eval(S, orc.to_bytes([w0, w1]))) == [w0 * (1 - w1) % R]


def test_lagrange(orc):
    rng = random.Random(24)
    for deg in (2, 3):
        coef = [rng.randrange(R) for _ in range(deg + 1)]
        poly = lambda x: sum(c * pow(x, i, R) for i, c in enumerate(coef)) % R
        ys = orc.to_bytes([poly(j) for j in range(deg + 1)])
        for at in [0, 1, deg, rng.randrange(R), R - 1]:
            assert orc.to_ints(orc.lagrange_eval(ys, orc.to_bytes([at])[0])) == [poly(at)]
