"""GPU parity: the field kernels against the CPU oracle, element by element,
bit-exact (integer work)."""
import random

import numpy as np
import pytest
import torch

from tests.pyref import R

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def zk():
    import paper_2404_16109_amd as zk
    assert torch.cuda.is_available()
    return zk


def _values(rng, count):
    edge = [0, 1, 2, R - 1, R - 2, (R - 1) // 2, 2 ** 254, 2 ** 128 - 1, 2 ** 64, 2 ** 32 - 1, 2 ** 32, 2 ** 256 % R,
            2 ** 512 % R, 0xFFFFFFFF << 32, R - 2 ** 32]
    return edge + [rng.randrange(R) for _ in range(count)]


def test_constants(zk):
    rc, mod, r1, r2, ninv = zk.fr_constants()
    assert rc == 0 and mod == R and r1 == 2 ** 256 % R and r2 == 2 ** 512 % R
    assert ninv == (-pow(R, -1, 2 ** 32)) % 2 ** 32


def test_roundtrip_and_binary_ops(zk, orc):
    rng = random.Random(1)
    a = _values(rng, 3000)            # several workgroups and a ragged tail
    b = list(reversed(_values(rng, 3000)))
    A, B = orc.to_bytes(a), orc.to_bytes(b)
    va, vb = zk.vec_from_bytes(A), zk.vec_from_bytes(B)
    assert np.array_equal(zk.vec_to_bytes(va), A)
    out = zk.Vec(len(a))
    for name in ("fr_add", "fr_sub", "fr_mul"):
        assert getattr(zk, name)(out, va, vb) == 0
        assert np.array_equal(zk.vec_to_bytes(out), getattr(orc, name)(A, B)), name
    # aliasing dst with an input
    assert zk.fr_mul(va, va, vb) == 0
    assert np.array_equal(zk.vec_to_bytes(va), orc.fr_mul(A, B))


def test_all_edge_pairs_multiply(zk, orc):
    rng = random.Random(2)
    edge = _values(rng, 0)
    a = [x for x in edge for _ in edge]
    b = [y for _ in edge for y in edge]
    A, B = orc.to_bytes(a), orc.to_bytes(b)
    out = zk.Vec(len(a))
    assert zk.fr_mul(out, zk.vec_from_bytes(A), zk.vec_from_bytes(B)) == 0
    assert np.array_equal(zk.vec_to_bytes(out), orc.fr_mul(A, B))


def test_scalar_ops(zk, orc):
    rng = random.Random(3)
    x, y = _values(rng, 700), _values(rng, 700)
    X, Y = orc.to_bytes(x), orc.to_bytes(y)
    vx, vy = zk.vec_from_bytes(X), zk.vec_from_bytes(Y)
    out = zk.Vec(len(x))
    for s in (0, 1, R - 1, rng.randrange(R)):
        sb = orc.to_bytes([s])[0]
        assert zk.fr_add_scalar(out, vx, s) == 0
        assert np.array_equal(zk.vec_to_bytes(out), orc.fr_axpy(X, sb))
        assert zk.fr_mul_scalar(out, vx, s) == 0
        assert np.array_equal(zk.vec_to_bytes(out), orc.fr_mul_scalar(X, sb))
        assert zk.fr_axpy(out, vx, s, vy) == 0
        assert np.array_equal(zk.vec_to_bytes(out), orc.fr_axpy(X, sb, Y))
    assert zk.fr_add_scalar(out, vx, R) == zk.ZK_E_BADARG   # scalar must be canonical


def test_signed_embedding(zk, orc):
    rng = np.random.default_rng(4)
    x = np.concatenate([np.array([0, 1, -1, 2 ** 31 - 1, -2 ** 31, 32767, -32768], dtype=np.int64),
                        rng.integers(-2 ** 31, 2 ** 31, 1000)])
    out = zk.Vec(len(x))
    assert zk.fr_from_i32(out, torch.from_numpy(x.astype(np.int32)).cuda()) == 0
    assert np.array_equal(zk.vec_to_bytes(out), orc.fr_from_i64(x))


def test_empty_and_bad_arguments(zk):
    e = zk.Vec(0)
    assert zk.fr_add(e, e, e) == 0
    a, b = zk.Vec(4), zk.Vec(3)
    assert zk.fr_add(a, a, b) == zk.ZK_E_BADARG


@pytest.mark.parametrize("n", [1, 2, 63, 256, 257, 1000, 1024, 1025, 4096, 4097, 16385, 70001, 300001])
def test_batch_inverse(zk, orc, n):
    rng = random.Random(10 + n)
    x = [rng.randrange(1, R) for _ in range(n)]
    x[0] = 1
    x[-1] = R - 1
    X = orc.to_bytes(x)
    rc_o, want = orc.fr_inv(X)
    out = zk.Vec(n)
    assert zk.fr_batch_inverse(out, zk.vec_from_bytes(X)) == 0 == rc_o
    got = zk.vec_to_bytes(out)
    assert np.array_equal(got, want)
    # a * a^-1 = 1 on every output
    assert orc.to_ints(orc.fr_mul(got, X)) == [1] * n


@pytest.mark.parametrize("n", [(1 << 22) + 4097, 5 * (1 << 20) + 3, (1 << 24) + 1])
def test_batch_inverse_long(zk, orc, n):
    """Lengths whose reduction takes one, two and three levels below the first, the
    last of them by whole workgroups with a ragged end.  Checked by the defining
    property x * x^-1 = 1 on every element (the product is the library's, pinned
    elsewhere against the oracle), and against the oracle on a sample."""
    rng = random.Random(n)
    raw = np.random.default_rng(n).integers(0, 256, size=(n, 32), dtype=np.uint8) & np.array([255] * 31 + [63], dtype=np.uint8)
    X = zk.vec_from_bytes(raw)
    out, prod = zk.Vec(n), zk.Vec(n)
    assert zk.fr_batch_inverse(out, X) == 0
    assert zk.fr_mul(prod, out, X) == 0
    got = zk.vec_to_bytes(prod)
    one = np.zeros(32, dtype=np.uint8)
    one[0] = 1
    assert np.array_equal(got, np.broadcast_to(one, (n, 32)))
    pick = sorted({0, 1, 255, 256, 4095, 4096, n - 1, n - 2, n - 4097} | {rng.randrange(n) for _ in range(200)})
    rc_o, want = orc.fr_inv(np.ascontiguousarray(raw[pick]))
    assert rc_o == 0 and np.array_equal(zk.vec_to_bytes(out)[pick], want)


def test_batch_inverse_two_levels_of_threads(zk, orc):
    """2^26 + 4097 elements: the level below the first is still too long for whole
    workgroups.  Inputs are small integers made on the device; every product
    x * x^-1 must be the field's one, compared on the device, and a sample of the
    inverses must equal the oracle's."""
    import torch
    n = (1 << 26) + 4097
    g = torch.Generator(device="cuda")
    g.manual_seed(26)
    ints = torch.randint(1, 2 ** 31 - 1, (n,), dtype=torch.int32, device="cuda", generator=g)
    X, out = zk.Vec(n), zk.Vec(n)
    assert zk.fr_from_i32(X, ints) == 0
    assert zk.fr_batch_inverse(out, X) == 0
    assert zk.fr_mul(X, out, X) == 0
    one = zk.Vec(1)
    assert zk.fr_from_i32(one, torch.ones(1, dtype=torch.int32, device="cuda")) == 0
    assert bool((X.data[:, :n] == one.data[:, :1]).all())
    pick = torch.tensor(sorted({0, 4095, 4096, n - 1, n - 4098} | {(i * 7919 * 4099) % n for i in range(100)}), device="cuda")
    sample = zk.Vec(len(pick))
    sample.data.copy_(out.data[:, pick])
    rc_o, want = orc.fr_inv(orc.to_bytes([int(v) for v in ints[pick].cpu()]))
    assert rc_o == 0 and np.array_equal(zk.vec_to_bytes(sample), want)


def test_batch_inverse_reports_zero(zk, orc):
    rng = random.Random(11)
    for n, pos in ((5, 2), (5000, 4999), (5000, 0), (70001, 33333)):
        x = [rng.randrange(1, R) for _ in range(n)]
        x[pos] = 0
        out = zk.Vec(n)
        assert zk.fr_batch_inverse(out, zk.vec_from_bytes(orc.to_bytes(x))) == zk.ZK_E_ZERO_DENOM


def test_sum(zk, orc):
    rng = random.Random(12)
    for n in (1, 100, 256, 5000, 300000):
        X = orc.to_bytes([rng.randrange(R) for _ in range(n)]) if n < 10000 else \
            np.frombuffer(rng.randbytes(32 * n), dtype=np.uint8).reshape(n, 32) & np.array([255] * 31 + [63], dtype=np.uint8)
        rc, got = zk.fr_sum(zk.vec_from_bytes(X))
        assert rc == 0 and [got] == orc.to_ints(orc.fr_sum(X)), n


@pytest.mark.parametrize("nvars", [0, 1, 3, 4, 5, 11, 14])
def test_eq_table_and_mle(zk, orc, nvars):
    rng = random.Random(20 + nvars)
    u = [rng.randrange(R) for _ in range(nvars)]
    U = orc.to_bytes(u) if nvars else np.zeros((0, 32), dtype=np.uint8)
    tab = zk.Vec(1 << nvars)
    assert zk.fr_eq_table(tab, u) == 0
    want = orc.eq_table(U) if nvars else orc.to_bytes([1])
    assert np.array_equal(zk.vec_to_bytes(tab), want)
    vals = [rng.randrange(R) for _ in range(1 << nvars)] if nvars <= 11 else None
    V = orc.to_bytes(vals) if vals else np.frombuffer(rng.randbytes(32 << nvars), dtype=np.uint8).reshape(-1, 32) & np.array([255] * 31 + [63], dtype=np.uint8)
    rc, got = zk.fr_mle_eval(zk.vec_from_bytes(V), u)
    expect = orc.to_ints(orc.mle_eval(V, U))[0] if nvars else orc.to_ints(V)[0]
    assert rc == 0 and got == expect
