"""The small-integer arithmetic of the device library (csrc/small_dev.h is plain
C++), built for the host with g++ and compared with Python integers: products of
a field element with a 32- or 64-bit integer accumulated without reduction, the
short Montgomery reduction, and the fold a + rho (b - a) of two small integers
straight into a reduced field element in Montgomery form."""
import ctypes
import os
import random
import subprocess
import tempfile

import numpy as np
import pytest

R = 0x73eda753299d7d483339d80809a1d80553bda402fffe5bfeffffffff00000001
MONT = pow(2, 256, R)
HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def lib():
    d = tempfile.mkdtemp(prefix="small_")
    so = os.path.join(d, "small_check.so")
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC",
                           os.path.join(HERE, "native", "small_check.cpp"), "-o", so])
    lib = ctypes.CDLL(so)
    lib.c_mac64.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64]
    lib.c_mac32.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32]
    lib.c_fold64.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
    lib.c_fold32.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p]
    return lib


def words(x, n):
    return np.array([(x >> (32 * i)) & 0xFFFFFFFF for i in range(n)], dtype=np.uint32)


def value(w):
    return sum(int(v) << (32 * i) for i, v in enumerate(w))


def ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def test_modulus_words():
    src = open(os.path.join(HERE, "..", "paper_2404_16109_amd", "csrc", "small_dev.h")).read()
    import re
    body = src.split("#define ZK_SMALL_R_WORDS")[1].split("}")[0]
    assert value([int(h, 16) for h in re.findall(r"0x([0-9a-fA-F]+)u", body)]) == R


def test_products_accumulate_exactly(lib):
    rng = random.Random(1)
    for _ in range(200):
        total = rng.randrange(2 ** 330)
        t = words(total, 11)
        for _ in range(rng.randrange(1, 6)):
            c = rng.choice([rng.randrange(R), R - 1, 2 ** 256 - 1, 0])
            if rng.random() < 0.5:
                m = rng.choice([rng.randrange(2 ** 32), 2 ** 32 - 1, 0])
                lib.c_mac32(ptr(t), ptr(words(c, 8)), m)
            else:
                m = rng.choice([rng.randrange(2 ** 64), 2 ** 64 - 1, 1 << 32, 0])
                lib.c_mac64(ptr(t), ptr(words(c, 8)), m)
            total += c * m
        assert value(t) == total and total < 2 ** 352


def test_short_reduction(lib):
    rng = random.Random(2)
    for steps, fn, nl in ((2, "c_reduce2", 11), (3, "c_reduce3", 12)):
        for _ in range(200):
            t = rng.choice([rng.randrange(R << (32 * steps)), (R << (32 * steps)) - 1, 0, R, rng.randrange(2 ** 64)])
            out = np.zeros(8, np.uint32)
            getattr(lib, fn)(ptr(words(t, nl)), ptr(out))
            assert value(out) == t * pow(2, -32 * steps, R) % R


def fold_consts(s, rho):
    """Montgomery forms, times 2^64, of s, -s, rho s, -rho s."""
    scale = MONT * pow(2, 64, R)
    vals = [s * scale % R, -s * scale % R, rho * s * scale % R, -rho * s * scale % R]
    return np.concatenate([words(v, 8) for v in vals])


def test_fold_of_small_integers(lib):
    rng = random.Random(3)
    edge64 = [0, 1, -1, 2 ** 62 - 1, -(2 ** 62 - 1)]
    edge32 = [0, 1, 2 ** 32 - 1]
    for _ in range(300):
        s, rho = rng.choice([1, rng.randrange(1, R)]), rng.choice([0, 1, rng.randrange(R), R - 1])
        k = fold_consts(s, rho)
        a = rng.choice(edge64 + [rng.randrange(-(2 ** 62) + 1, 2 ** 62)])
        b = rng.choice(edge64 + [rng.randrange(-(2 ** 62) + 1, 2 ** 62)])
        out = np.zeros(8, np.uint32)
        lib.c_fold64(a, b, ptr(k), ptr(out))
        assert value(out) == (a + rho * (b - a)) * s * MONT % R
        a = rng.choice(edge32 + [rng.randrange(2 ** 32)])
        b = rng.choice(edge32 + [rng.randrange(2 ** 32)])
        lib.c_fold32(a, b, ptr(k), ptr(out))
        assert value(out) == (a + rho * (b - a)) * s * MONT % R


def test_pair_of_columns_combined_and_folded(lib):
    """x + rho y, and the fold of two such entries by a challenge, for signed 32-bit columns."""
    lib.c_combine32.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
    lib.c_fold_combined.argtypes = [ctypes.c_int32] * 4 + [ctypes.c_void_p, ctypes.c_void_p]
    rng = random.Random(4)
    scale = MONT * pow(2, 64, R)
    edge = [0, 1, -1, 2 ** 31 - 1, -(2 ** 31)]
    pick = lambda: rng.choice(edge + [rng.randrange(-(2 ** 31), 2 ** 31)])
    for _ in range(300):
        rho, c = rng.choice([0, 1, rng.randrange(R), R - 1]), rng.choice([0, 1, rng.randrange(R), R - 1])
        k = np.concatenate([words(v * scale % R, 8) for v in (1, -1, rho, -rho)])
        x, y = pick(), pick()
        out = np.zeros(8, np.uint32)
        lib.c_combine32(x, y, ptr(k), ptr(out))
        assert value(out) == (x + rho * y) * MONT % R
        k4 = np.concatenate([words(v * scale % R, 8) for v in (1, -1, c, -c, rho, -rho, rho * c, -rho * c)])
        x1, y1 = pick(), pick()
        lib.c_fold_combined(x, y, x1, y1, ptr(k4), ptr(out))
        s0, s1 = x + rho * y, x1 + rho * y1
        assert value(out) == (s0 + c * (s1 - s0)) * MONT % R
