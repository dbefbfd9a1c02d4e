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


def test_mul_add_is_product_plus_addend(lib):
    rng = random.Random(8)
    inv = pow(2, -261, R)
    cases = []
    for _ in range(300):  # the fold: a padded difference times the challenge, plus an entry below 17 r
        cases.append((lazy_limbs(rng, 3 * 2 ** 29, 2 ** 29), limbs_of(rng.randrange(R)), limbs_of(rng.randrange(17 * R))))
    cases.append((arr([3 * 2 ** 29 - 1] * 8 + [2 ** 29]), arr([M29] * 8 + [0x73eda7]), arr([M29] * 8 + [0x7b2ec8])))
    for a, b, c in cases:
        out = np.zeros(9, np.uint32)
        lib.c_mul_add(ptr(a), ptr(b), ptr(c), ptr(out))
        va, vb, vc, vo = value_of(a), value_of(b), value_of(c), value_of(out)
        assert vo % R == (va * vb * inv + vc) % R
        assert vo < va * vb // 2 ** 261 + R + 1 + vc
        assert all(int(v) <= M29 for v in out[:8])


def test_shrink(lib):
    rng = random.Random(10)
    for x in [0, 1, R, 272 * R, 2 ** 264 - 1] + [rng.randrange(2 ** 264) for _ in range(200)]:
        out = np.zeros(9, np.uint32)
        lib.c_shrink(ptr(limbs_of(x)), ptr(out))
        vo = value_of(out)
        assert vo % R == x % R and vo < x * pow(2, 261, R) // 2 ** 261 + R + 1 and all(int(v) <= M29 for v in out[:8])
        assert vo < 9 * R


def _round29_thread(lib, entries, weights, r261, beta, want_peak=True):
    pairs = len(weights)
    e = np.concatenate([np.concatenate(p) for p in entries]).astype(np.uint32)
    w = np.concatenate(weights).astype(np.uint32)
    folded = np.zeros(36 * pairs, np.uint32)
    out = np.zeros(27, np.uint32)
    peak = ctypes.c_uint64(0)
    lib.c_round29_thread(pairs, ptr(e), ptr(w), ptr(limbs_of(r261)), ptr(limbs_of(beta)), ptr(folded), ptr(out),
                         ctypes.byref(peak) if want_peak else None)
    return folded.reshape(pairs, 4, 9), out.reshape(3, 9), peak.value


def _check_round29_thread(lib, entries, weights, r261, beta):
    """The whole per-thread schedule of the large folding rounds against Python integers: the four folds of
    every pair, the three sums, and every bound the kernel's sums across lanes rely on."""
    inv = pow(2, -261, R)
    folded, out, peak = _round29_thread(lib, entries, weights, r261, beta)
    q0 = qinf = sA0 = 0
    for j, (pair, w) in enumerate(zip(entries, weights)):
        y = [value_of(v) for v in pair]
        want = [(y[0] + (y[2] - y[0]) * r261 * inv) % R, (y[1] + (y[3] - y[1]) * r261 * inv) % R,
                (y[4] + (y[6] - y[4]) * r261 * inv) % R, (y[5] + (y[7] - y[5]) * r261 * inv) % R]
        got = [value_of(folded[j][q]) for q in range(4)]
        assert [g % R for g in got] == want
        # a fold adds less than 2 r to the entry it starts from, and leaves normalized limbs
        for g, start in zip(got, (y[0], y[1], y[4], y[5])):
            assert g < start + 2 * R
        assert all(int(v) <= M29 for q in range(4) for v in folded[j][q][:8])
        a0, a1, s0, s1 = want
        wv = value_of(w)
        q0 += (a0 * wv * inv) * (s0 + beta)
        qinf += ((a1 - a0) * wv * inv) * (s1 - s0)
        sA0 += a0
    got = [value_of(out[q]) for q in range(3)]
    assert got[0] % R == q0 * inv % R and got[1] % R == qinf * inv % R and got[2] % R == sA0 % R
    # what the sums over a wavefront (64 lanes: below 2^264, about 565 r), the shrink after it and the sum over the
    # workgroup's wavefronts need
    assert got[0] < 1.2 * R and got[1] < 2.6 * R and got[2] < 6.3 * R
    assert all(int(v) <= M29 for q in range(3) for v in out[q][:8])
    assert peak < 2 ** 32 - 2 ** 29          # no lazy limb came near wrapping between two normalizations
    return peak


def test_round29_thread_schedule_at_its_bounds(lib):
    """As many pairs per thread as the prover ever gives one (22), entries at the bound eight lazy rounds can reach
    (just below 17 r) with every limb full, the largest weight, challenge and beta: the worst case for every
    accumulator of the schedule."""
    top17 = (17 * R - 1) >> 232
    full = arr([M29] * 8 + [top17 - 1])         # all limbs full, value just below 17 r
    assert 16 * R < value_of(full) < 17 * R
    zero = arr([0] * 9)
    rmax = arr([(R - 1 >> (29 * i)) & M29 for i in range(8)] + [(R - 1) >> 232])
    worst = 0
    for entries_of_pair in ([full] * 8,                                   # everything at the bound
                            [zero, full, full, zero, full, zero, zero, full],   # differences at their extremes
                            [full, zero, zero, full, zero, full, full, zero]):
        for r261 in (R - 1, 1, pow(2, 261, R)):
            peak = _check_round29_thread(lib, [entries_of_pair] * 22, [rmax] * 22, r261, R - 1)
            worst = max(worst, peak)
    assert worst > 2 ** 31                      # the test does reach the region the bound is about
    rng = random.Random(11)
    for pairs in (1, 2, 3, 4, 7, 8, 16, 21, 22):
        entries = [[limbs_of(rng.randrange(17 * R)) for _ in range(8)] for _ in range(pairs)]
        weights = [limbs_of(rng.randrange(R)) for _ in range(pairs)]
        _check_round29_thread(lib, entries, weights, rng.randrange(R), rng.randrange(R))


def test_round29_eight_lazy_rounds_in_a_row(lib):
    """Entries that start below r stay below 17 r through eight folds in a row (what the prover runs before it
    writes reduced words again), with the challenge that makes every fold add the most."""
    rng = random.Random(12)
    vals = [limbs_of(R - 1 - rng.randrange(1000)) for _ in range(8)]
    for rnd in range(8):
        folded, out, _ = _round29_thread(lib, [vals], [limbs_of(R - 1)], R - 1, R - 1, want_peak=False)
        nxt = [folded[0][q].copy() for q in range(4)]
        assert all(value_of(v) < (1 + 2 * (rnd + 1)) * R for v in nxt)
        vals = [nxt[0], nxt[1], nxt[2], nxt[3], nxt[2], nxt[3], nxt[0], nxt[1]]
    assert max(value_of(v) for v in vals) < 17 * R


def _round01_thread(lib, entries, weights):
    quads = len(weights)
    e = np.concatenate([np.concatenate(q) for q in entries]).astype(np.uint32)
    w = np.concatenate(weights).astype(np.uint32)
    out = np.zeros(81, np.uint32)
    peak = ctypes.c_uint64(0)
    lib.c_round01_thread(quads, ptr(e), ptr(w), ptr(out), ctypes.byref(peak))
    return out.reshape(9, 9), peak.value


def _check_round01_thread(lib, entries, weights):
    """The per-thread schedule of the first pass when it serves two rounds, against Python integers: the five sums of
    products and the four sums of A, and every bound the kernel's sums across lanes rely on."""
    inv = pow(2, -261, R)
    out, peak = _round01_thread(lib, entries, weights)
    want = [0] * 9
    for quad, w in zip(entries, weights):
        a = [value_of(v) for v in quad[:4]]
        s = [value_of(v) for v in quad[4:]]
        wv = value_of(w)
        B = lambda x, y: x * wv * inv * y
        want[0] += B(a[2] - a[0], s[2] - s[0])
        want[1] += B(a[3] - a[1], s[3] - s[1])
        want[2] += B(a[1] - a[0], s[1] - s[0])
        want[3] += B(a[3] - a[2], s[3] - s[2])
        want[4] += B(a[3] - a[1] - a[2] + a[0], s[3] - s[1] - s[2] + s[0])
        for c in range(4):
            want[5 + c] += a[c]
    got = [value_of(out[q]) for q in range(9)]
    for q in range(9):
        assert got[q] % R == (want[q] * inv if q < 5 else want[q]) % R, q
    # what the sums over a wavefront (64 lanes) and then over four wavefronts need
    assert all(g < 2 * R for g in got) and all(int(v) <= M29 for q in range(9) for v in out[q][:8])
    assert peak <= 2 ** 32 - 8               # no lazy limb wrapped before a normalization
    return peak


def test_round01_thread_schedule_at_its_bounds(lib):
    """Sixteen quads per thread (the most the prover gives one), every entry the largest a reduced element can be or
    zero, so that every difference is at an extreme, with the largest weight: the worst case for the accumulators of
    the first pass."""
    rmax = limbs_of(R - 1)
    zero = arr([0] * 9)
    worst = 0
    patterns = [[rmax] * 8,
                [zero, rmax, rmax, zero, rmax, zero, zero, rmax],
                [rmax, zero, zero, rmax, zero, rmax, rmax, zero],
                [zero, zero, rmax, rmax, rmax, rmax, zero, zero],
                [rmax, zero, rmax, zero, zero, rmax, zero, rmax]]
    for pat in patterns:
        worst = max(worst, _check_round01_thread(lib, [pat] * 16, [rmax] * 16), _check_round01_thread(lib, [pat] * 7, [rmax] * 7),
                    _check_round01_thread(lib, [pat] * 14, [rmax] * 14))
    assert worst > 2 ** 31                   # the test does reach the region the bound is about
    rng = random.Random(21)
    for quads in (1, 2, 3, 5, 8, 9, 15, 16):
        entries = [[limbs_of(rng.randrange(R)) for _ in range(8)] for _ in range(quads)]
        weights = [limbs_of(rng.randrange(R)) for _ in range(quads)]
        _check_round01_thread(lib, entries, weights)


def test_round01_sums_give_the_second_round(lib):
    """With A_c (S_c + beta) = 1 for every entry, the second round's sums after a first challenge r are the polynomials
    in r that the prover forms from the pass's sums: checked here on Python integers against folding first."""
    rng = random.Random(22)
    quads = 6
    beta = rng.randrange(R)
    S = [[rng.randrange(R) for _ in range(4)] for _ in range(quads)]
    A = [[pow(beta + s, -1, R) for s in q] for q in S]
    w = [rng.randrange(R) for _ in range(quads)]
    wsum = sum(w) % R
    B = lambda f: sum(w[j] * f(A[j], S[j]) for j in range(quads)) % R
    c20 = B(lambda a, s: (a[2] - a[0]) * (s[2] - s[0]))
    c21 = B(lambda a, s: (a[3] - a[1]) * (s[3] - s[1]))
    qd = B(lambda a, s: (a[1] - a[0]) * (s[1] - s[0]))
    T = B(lambda a, s: (a[3] - a[2]) * (s[3] - s[2]))
    qe = B(lambda a, s: (a[3] - a[1] - a[2] + a[0]) * (s[3] - s[1] - s[2] + s[0]))
    r = rng.randrange(R)
    fold = lambda y: ((y[0] + r * (y[2] - y[0])) % R, (y[1] + r * (y[3] - y[1])) % R)
    Af, Sf = [fold(a) for a in A], [fold(s) for s in S]
    q0 = sum(w[j] * Af[j][0] * (Sf[j][0] + beta) for j in range(quads)) % R
    q1 = sum(w[j] * Af[j][1] * (Sf[j][1] + beta) for j in range(quads)) % R
    qinf = sum(w[j] * (Af[j][1] - Af[j][0]) * (Sf[j][1] - Sf[j][0]) for j in range(quads)) % R
    t = r * (1 - r)
    assert q0 == (wsum - t * c20) % R and q1 == (wsum - t * c21) % R     # the weights of a whole round sum to one
    assert qinf == (qd + r * (T - qd - qe) + r * r * qe) % R


def test_mul3_add_is_three_products_under_one_reduction(lib):
    rng = random.Random(24)
    inv = pow(2, -261, R)
    full = value_of([M29] * 8 + [(42 * R) >> 232])   # every limb full, value about 42 r: the largest a normalized difference gets
    for trial in range(60):
        if trial == 0:
            vals = [full, R - 1, full, R - 1, full, R - 1, value_of([M29] * 8 + [(17 * R) >> 232])]
        else:
            vals = [rng.randrange(42 * R), rng.randrange(R), rng.randrange(42 * R), rng.randrange(R),
                    rng.randrange(42 * R), rng.randrange(R), rng.randrange(17 * R)]
        out = np.zeros(9, np.uint32)
        lib.c_mul3_add(ptr(np.concatenate([limbs_of(v) for v in vals])), ptr(out))
        prod = vals[0] * vals[1] + vals[2] * vals[3] + vals[4] * vals[5]
        got = value_of(out)
        assert got % R == (prod * inv + vals[6]) % R
        assert got < prod // 2 ** 261 + R + vals[6] + 1 and all(int(v) <= M29 for v in out[:8])


def test_fold2_binds_two_variables(lib):
    rng = random.Random(23)
    inv = pow(2, -261, R)
    rmax = R - 1
    for trial in range(60):
        if trial < 4:   # entries at their extremes, so that every difference is, with the largest challenges
            y = [[rmax, rmax, rmax, rmax], [0, rmax, rmax, 0], [rmax, 0, 0, rmax], [0, 0, 0, rmax]][trial]
            r0 = r1 = rmax
        else:
            y = [rng.randrange(R) for _ in range(4)]
            r0, r1 = rng.randrange(R), rng.randrange(R)
        r01 = r0 * r1 * inv % R       # the product of the two, again times 2^261
        out = np.zeros(9, np.uint32)
        lib.c_fold2(ptr(np.concatenate([limbs_of(v) for v in y])), ptr(limbs_of(r0)), ptr(limbs_of(r1)), ptr(limbs_of(r01)),
                    ptr(out))
        # bind x_0 (entries y_00, y_10 and y_01, y_11), then x_1
        lo = y[0] + (y[2] - y[0]) * r0 * inv
        hi = y[1] + (y[3] - y[1]) * r0 * inv
        assert value_of(out) % R == (lo + (hi - lo) * r1 * inv) % R
        # within what two single folds may add: below its first entry + 2.8 r, normalized
        assert value_of(out) < y[0] + 2.8 * R and all(int(v) <= M29 for v in out[:8])
