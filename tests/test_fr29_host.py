"""The 29-bit-limb field arithmetic of the device library (csrc/fr29_dev.h is
plain C++), built for the host with g++ and compared with Python integers: layout
changes, lazy differences, Montgomery products by 2^261, unreduced sums of
products, and the way back to the canonical representative, each at the limb
and value bounds its comment states."""
import ctypes
import os
import random
import subprocess
import tempfile

import numpy as np
import pytest

R = 0x73eda753299d7d483339d80809a1d80553bda402fffe5bfeffffffff00000001
M29 = (1 << 29) - 1
HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def lib():
    d = tempfile.mkdtemp(prefix="fr29_")
    so = os.path.join(d, "fr29_check.so")
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC",
                           os.path.join(HERE, "native", "fr29_check.cpp"), "-o", so])
    return ctypes.CDLL(so)


def arr(vals):
    return np.array(vals, dtype=np.uint32)


def ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def limbs_of(x, n=9):
    out = [(x >> (29 * i)) & M29 for i in range(n - 1)]
    out.append(x >> (29 * (n - 1)))
    assert out[-1] < 2 ** 32
    return arr(out)


def value_of(l):
    return sum(int(v) << (29 * i) for i, v in enumerate(l))


def words_of(x):
    return arr([(x >> (32 * i)) & 0xFFFFFFFF for i in range(8)])


def words_value(w):
    return sum(int(v) << (32 * i) for i, v in enumerate(w))


def lazy_limbs(rng, limb_bound, top_bound):
    return arr([rng.randrange(limb_bound) for _ in range(8)] + [rng.randrange(top_bound)])


def test_constants():
    import re
    src = open(os.path.join(HERE, "..", "paper_2404_16109_amd", "csrc", "fr29_dev.h")).read()

    def macro(name):
        body = src.split("#define " + name)[1].split("}")[0]
        return [int(h, 16) for h in re.findall(r"0x([0-9a-fA-F]+)u", body)]

    assert value_of(macro("ZK_R29_LIMBS")) == R
    assert all(v <= M29 for v in macro("ZK_R29_LIMBS"))
    assert value_of(macro("ZK_ONE261_LIMBS")) == pow(2, 261, R)
    pad = macro("ZK_SUBPAD_LIMBS")
    assert value_of(pad) == 40 * R
    assert all(v >= M29 for v in pad[:8]) and all(v < 2 ** 31 for v in pad)
    pad4 = macro("ZK_SUBPAD4_LIMBS")
    assert value_of(pad4) == 4 * R
    assert all(v >= M29 for v in pad4[:8]) and all(v < 2 ** 31 for v in pad4)


def test_unpack_pack_roundtrip(lib):
    rng = random.Random(1)
    for x in [0, 1, R - 1, 2 ** 256 - 1, 2 ** 255] + [rng.randrange(2 ** 256) for _ in range(200)]:
        out = np.zeros(9, np.uint32)
        lib.c_unpack(ptr(words_of(x)), ptr(out))
        assert value_of(out) == x and all(int(v) <= M29 for v in out)
        w = np.zeros(8, np.uint32)
        lib.c_pack(ptr(out), ptr(w))
        assert words_value(w) == x


def test_normalize(lib):
    rng = random.Random(2)
    for _ in range(200):
        l = lazy_limbs(rng, 2 ** 32 - 16, 2 ** 28)
        out = np.zeros(9, np.uint32)
        lib.c_normalize(ptr(l), ptr(out))
        assert value_of(out) == value_of(l)
        assert all(int(v) <= M29 for v in out[:8])


def test_sub_is_difference_mod_r_without_negative_limbs(lib):
    rng = random.Random(3)
    for _ in range(300):
        a = lazy_limbs(rng, 2 ** 30, 2 ** 28)
        b = limbs_of(rng.randrange(39 * R))  # normalized, below 39.99 r
        if rng.random() < 0.2:
            b = limbs_of(int(39.98 * R))
        if rng.random() < 0.1:
            b = arr([M29] * 8 + [0x121d2223])  # the largest subtrahend the padding allows
        out = np.zeros(9, np.uint32)
        lib.c_sub(ptr(a), ptr(b), ptr(out))
        assert value_of(out) == value_of(a) - value_of(b) + 40 * R
        assert all(int(o) < int(x) + 2 ** 30 for o, x in zip(out, a))


def test_sub_small(lib):
    rng = random.Random(7)
    for _ in range(300):
        a = limbs_of(rng.randrange(2 * R))
        b = limbs_of(rng.randrange(2 * R)) if rng.random() < 0.9 else arr([M29] * 8 + [0x01cfb69c])
        out = np.zeros(9, np.uint32)
        lib.c_sub_small(ptr(a), ptr(b), ptr(out))
        assert value_of(out) == value_of(a) - value_of(b) + 4 * R
        assert all(int(o) < 2 ** 29 + 2 ** 30 for o in out)


def test_mul_is_montgomery_product(lib):
    rng = random.Random(4)
    cases = []
    for _ in range(300):  # normalized operands
        cases.append((limbs_of(rng.randrange(2 ** 258)), limbs_of(rng.randrange(2 ** 258))))
    for _ in range(300):  # a lazy difference times a normalized factor
        cases.append((lazy_limbs(rng, 3 * 2 ** 29, 2 ** 29), limbs_of(rng.randrange(R))))
    for _ in range(300):  # two lazy sums
        cases.append((lazy_limbs(rng, 2 ** 30, 2 ** 27), lazy_limbs(rng, 2 ** 30, 2 ** 27)))
    # the largest limbs each case allows
    cases.append((arr([3 * 2 ** 29 - 1] * 8 + [2 ** 29]), arr([M29] * 8 + [0x73eda7])))
    cases.append((arr([2 ** 30 - 1] * 8 + [2 ** 27]), arr([2 ** 30 - 1] * 8 + [2 ** 27])))
    inv = pow(2, -261, R)
    for a, b in cases:
        out = np.zeros(9, np.uint32)
        lib.c_mul(ptr(a), ptr(b), ptr(out))
        va, vb, vo = value_of(a), value_of(b), value_of(out)
        assert vo % R == va * vb * inv % R
        assert vo < va * vb // 2 ** 261 + R + 1
        assert all(int(v) <= M29 for v in out[:8])


def test_wide_sums_of_products(lib):
    rng = random.Random(5)
    inv = pow(2, -261, R)
    for _ in range(50):
        w = np.zeros(18, np.uint32)
        want = 0
        for rep in range(16):
            a = limbs_of(rng.randrange(2 ** 256))
            b = lazy_limbs(rng, 3 * 2 ** 29, 2 ** 29)
            lib.c_wide_mac(ptr(w), ptr(a), ptr(b))
            want += value_of(a) * value_of(b)
            if rep % 8 == 7:
                lib.c_wide_normalize(ptr(w))
                assert all(int(v) <= M29 for v in w[:17])
            assert sum(int(v) << (29 * i) for i, v in enumerate(w)) == want
        out = np.zeros(9, np.uint32)
        lib.c_wide_reduce(ptr(w), ptr(out))
        vo = value_of(out)
        assert vo % R == want * inv % R and vo < want // 2 ** 261 + R + 1
        assert all(int(v) <= M29 for v in out[:8])
        c = np.zeros(8, np.uint32)
        lib.c_canonical_big(ptr(out), ptr(c))
        assert words_value(c) == vo % R


def test_canonical(lib):
    rng = random.Random(6)
    for x in [0, 1, R - 1, R, R + 1, 2 * R, 2 ** 261 - 1] + [rng.randrange(2 ** 261) for _ in range(300)]:
        c = np.zeros(8, np.uint32)
        lib.c_canonical(ptr(limbs_of(x)), ptr(c))
        assert words_value(c) == x % R
    for _ in range(300):
        x = rng.randrange(2 ** 264)
        c = np.zeros(8, np.uint32)
        lib.c_canonical_big(ptr(limbs_of(x)), ptr(c))
        assert words_value(c) == x % R
