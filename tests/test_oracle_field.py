"""Pins of the oracle's field arithmetic against Python's big integers and the
closed forms that fix the field (no GPU)."""
import random

import numpy as np
import pytest

from tests.pyref import R, Z


def _edge_and_random(rng, count):
    edge = [0, 1, 2, R - 1, R - 2, (R - 1) // 2, (R + 1) // 2, 2 ** 254, 2 ** 128 - 1, 2 ** 64, 2 ** 64 - 1,
            2 ** 32, 2 ** 256 % R, 2 ** 512 % R]
    return edge + [rng.randrange(R) for _ in range(count)]


def test_modulus_is_the_curve_order(orc):
    lines = dict(l.split() for l in open("tests/golden/bls12_381_fr.txt") if l.strip() and not l.startswith("#"))
    assert int(lines["z"], 16) == Z
    assert int(lines["r"], 16) == Z ** 4 - Z ** 2 + 1 == R
    assert orc.modulus() == R
    assert R.bit_length() == 255
    assert (R - 1) % 2 ** 32 == 0 and (R - 1) % 2 ** 33 != 0


def test_modulus_is_prime():
    # Miller-Rabin with fixed and random bases
    d, s = R - 1, 0
    while d % 2 == 0:
        d //= 2
        s += 1
    rng = random.Random(7)
    for a in [2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37] + [rng.randrange(2, R - 1) for _ in range(20)]:
        x = pow(a, d, R)
        if x in (1, R - 1):
            continue
        for _ in range(s - 1):
            x = x * x % R
            if x == R - 1:
                break
        else:
            pytest.fail("composite witness %d" % a)


def test_barrett_constant(orc):
    assert orc.barrett_mu() == 2 ** 512 // R


def test_add_sub_mul_against_python(orc):
    rng = random.Random(11)
    vals = _edge_and_random(rng, 300)
    a = vals + [rng.choice(vals) for _ in range(300)]
    b = list(reversed(vals)) + [rng.choice(vals) for _ in range(300)]
    n = min(len(a), len(b))
    a, b = a[:n], b[:n]
    A, B = orc.to_bytes(a), orc.to_bytes(b)
    assert orc.to_ints(orc.fr_add(A, B)) == [(x + y) % R for x, y in zip(a, b)]
    assert orc.to_ints(orc.fr_sub(A, B)) == [(x - y) % R for x, y in zip(a, b)]
    assert orc.to_ints(orc.fr_mul(A, B)) == [(x * y) % R for x, y in zip(a, b)]


def test_mul_extremes(orc):
    # all pairs of edge values, including (r-1)^2 = 1
    rng = random.Random(5)
    edge = _edge_and_random(rng, 0)
    a = [x for x in edge for _ in edge]
    b = [y for _ in edge for y in edge]
    assert orc.to_ints(orc.fr_mul(orc.to_bytes(a), orc.to_bytes(b))) == [(x * y) % R for x, y in zip(a, b)]
    assert orc.to_ints(orc.fr_mul(orc.to_bytes([R - 1]), orc.to_bytes([R - 1]))) == [1]


def test_wide_reduction(orc):
    rng = random.Random(3)
    cases = [b"\x00" * 64, b"\xff" * 64, (R * R - 1).to_bytes(64, "big"), (2 ** 511).to_bytes(64, "big")]
    cases += [rng.randbytes(64) for _ in range(200)]
    for c in cases:
        assert orc.to_ints(orc.fr_from_be512(c)) == [int.from_bytes(c, "big") % R]


def test_inverse_and_fermat(orc):
    rng = random.Random(13)
    vals = [1, 2, R - 1, R - 2, 2 ** 256 % R] + [rng.randrange(1, R) for _ in range(40)]
    rc, inv = orc.fr_inv(orc.to_bytes(vals), threads=4)
    assert rc == orc.OK
    assert orc.to_ints(inv) == [pow(v, -1, R) for v in vals]
    assert orc.to_ints(orc.fr_mul(inv, orc.to_bytes(vals))) == [1] * len(vals)
    for v in vals[:8]:
        assert orc.to_ints(orc.fr_pow(orc.to_bytes([v])[0], R - 1)) == [1]
        e = rng.randrange(2 ** 256)
        assert orc.to_ints(orc.fr_pow(orc.to_bytes([v])[0], e)) == [pow(v, e, R)]
    rc, _ = orc.fr_inv(orc.to_bytes([3, 0, 5]))
    assert rc == orc.E_ZERO_DENOM


def test_ring_axioms(orc):
    rng = random.Random(17)
    n = 200
    a, b, c = ([rng.randrange(R) for _ in range(n)] for _ in range(3))
    A, B, C = orc.to_bytes(a), orc.to_bytes(b), orc.to_bytes(c)
    left = orc.fr_mul(A, orc.fr_add(B, C))
    right = orc.fr_add(orc.fr_mul(A, B), orc.fr_mul(A, C))
    assert np.array_equal(left, right)
    assert np.array_equal(orc.fr_mul(orc.fr_mul(A, B), C), orc.fr_mul(A, orc.fr_mul(B, C)))
    assert np.array_equal(orc.fr_sub(orc.fr_add(A, B), B), A)


def test_signed_embedding(orc):
    xs = np.array([0, 1, -1, 127, -128, 32767, -32768, 2 ** 31 - 1, -2 ** 31, 2 ** 62, -2 ** 62,
                   np.iinfo(np.int64).max, np.iinfo(np.int64).min], dtype=np.int64)
    got = orc.to_ints(orc.fr_from_i64(xs))
    assert got == [int(x) % R for x in xs]
    neg = orc.fr_from_i64(-xs[:-1])
    assert orc.to_ints(orc.fr_add(orc.fr_from_i64(xs[:-1]), neg)) == [0] * (len(xs) - 1)


def test_montgomery_constants_via_oracle(orc):
    # R_mont = 2^256: the constants the device library works with, recomputed
    # through the oracle's own arithmetic and compared with Python's.
    two = orc.to_bytes([2])[0]
    assert orc.to_ints(orc.fr_pow(two, 256)) == [2 ** 256 % R]
    assert orc.to_ints(orc.fr_pow(two, 512)) == [2 ** 512 % R]
    assert (-pow(R, -1, 2 ** 32)) % 2 ** 32 == 0xFFFFFFFF


def test_scalar_ops(orc):
    rng = random.Random(19)
    x = [rng.randrange(R) for _ in range(50)]
    y = [rng.randrange(R) for _ in range(50)]
    s = rng.randrange(R)
    sb = orc.to_bytes([s])[0]
    assert orc.to_ints(orc.fr_axpy(orc.to_bytes(x), sb, orc.to_bytes(y), threads=3)) == [(a + s * b) % R for a, b in zip(x, y)]
    assert orc.to_ints(orc.fr_axpy(orc.to_bytes(x), sb)) == [(a + s) % R for a in x]
    assert orc.to_ints(orc.fr_mul_scalar(orc.to_bytes(x), sb)) == [(a * s) % R for a in x]
    assert orc.to_ints(orc.fr_sum(orc.to_bytes(x))) == [sum(x) % R]
    assert orc.all_canonical(orc.to_bytes(x))
    bad = orc.to_bytes([1])
    bad[0] = np.frombuffer(R.to_bytes(32, "little"), dtype=np.uint8)
    assert not orc.all_canonical(bad)
