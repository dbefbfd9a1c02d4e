"""GPU parity of the sumcheck that links zkAttn's tensors (Protocol 2, last step):
the device library's proof must equal the oracle's byte for byte, for every
supported number of segments and for degenerate shapes; a witness that breaks a
relation is refused; the device verifier recomputes the stated values from the
tensors."""
import random

import numpy as np
import pytest
import torch

from tests.test_oracle_link import make_witness

pytestmark = pytest.mark.gpu
R = 0x73eda753299d7d483339d80809a1d80553bda402fffe5bfeffffffff00000001


@pytest.fixture(scope="module")
def zk():
    import paper_2404_16109_amd as zk
    assert torch.cuda.is_available()
    return zk


def to_device(zk, orc, w):
    Zp, X, Y, Yk, yhat, bases = w
    v = lambda a: zk.vec_from_bytes(orc.to_bytes(a))
    return v(Zp), [v(a) for a in X], v(Y), [v(a) for a in Yk], v(yhat), bases


def oracle_proof(orc, seed, w, rows, cols):
    Zp, X, Y, Yk, yhat, bases = w
    to = orc.to_bytes
    return orc.zkattn_link_prove(seed, to(Zp), [to(a) for a in X], to(Y), [to(a) for a in Yk], to(yhat), to(bases), rows, cols)


@pytest.mark.parametrize("rows,cols,K,digit_bits", [
    (1, 1, 2, 4), (1, 2, 2, 4), (2, 1, 1, 4), (4, 4, 3, 3), (1, 1024, 2, 8), (1024, 1, 2, 8), (8, 512, 2, 8),
    (64, 64, 1, 8), (32, 128, 3, 5), (512, 2, 2, 8), (16, 4096, 2, 8)])
def test_proof_equals_oracle(zk, orc, rows, cols, K, digit_bits):
    rng = random.Random(rows * 131 + cols * 7 + K)
    w = make_witness(rng, rows, cols, K, digit_bits=digit_bits, small_tables=rows * cols > 4096)
    seed = rng.randbytes(32)
    rc_o, want, point = oracle_proof(orc, seed, w, rows, cols)
    assert rc_o == 0
    Zp, X, Y, Yk, yhat, bases = to_device(zk, orc, w)
    rc, got = zk.zkattn_link_prove(seed, Zp, X, Y, Yk, yhat, bases, rows, cols)
    assert rc == zk.ZK_OK
    assert len(got) == len(want) == zk.zkattn_link_proof_bytes(rows, cols, K)
    assert got == want
    # inputs are left as they were
    assert np.array_equal(zk.vec_to_bytes(Y), orc.to_bytes(w[2])) and np.array_equal(zk.vec_to_bytes(X[K - 1]), orc.to_bytes(w[1][K - 1]))
    rc, claims = zk.zkattn_link_verify(seed, got, rows, cols, bases, Zp=Zp, X=X, Y=Y, Yk=Yk, yhat=yhat)
    assert rc == zk.ZK_OK and claims["v"] == orc.to_ints(point)
    assert orc.zkattn_link_verify(seed, got, rows, cols, orc.to_bytes(bases)) == 0


def test_attention_shaped_instance(zk, orc):
    """Two 16-bit digits with bases 1 and 2^16 and table outputs of the size of the
    fifth workload's, on 256 rows of 2048 scores (the workload's row length)."""
    rng = random.Random(5)
    rows, cols, K = 256, 2048, 2
    D = rows * cols
    gen = np.random.default_rng(5)
    x0 = gen.integers(0, 1 << 16, D)
    x1 = gen.integers(0, 13, D)
    t0 = gen.integers(1, 1 << 16, 1 << 16)
    t1 = gen.integers(0, 1 << 16, 1 << 16)
    y0, y1 = t0[x0], t1[x1]
    y = y0 * y1
    zp = -(x0 + (x1 << 16))
    yhat = y.reshape(rows, cols).sum(axis=1)
    to = lambda a: orc.fr_from_i64(np.asarray(a, dtype=np.int64))
    bases = [1, 1 << 16]
    seed = rng.randbytes(32)
    rc_o, want, _ = orc.zkattn_link_prove(seed, to(zp), [to(x0), to(x1)], to(y), [to(y0), to(y1)], to(yhat),
                                          orc.to_bytes(bases), rows, cols)
    assert rc_o == 0
    v = zk.vec_from_bytes
    dev = (v(to(zp)), [v(to(x0)), v(to(x1))], v(to(y)), [v(to(y0)), v(to(y1))], v(to(yhat)))
    rc, got = zk.zkattn_link_prove(seed, dev[0], dev[1], dev[2], dev[3], dev[4], bases, rows, cols)
    assert rc == zk.ZK_OK and got == want


def small_witness(gen, rows, cols, K, digit_bits, out_bits):
    """The relations' tensors as integers: digits, per-segment tables of out_bits-bit outputs,
    their product, the negated recomposed score and the row sums."""
    D = rows * cols
    bases = [1 << (digit_bits * k) for k in range(K)]
    X = [gen.integers(0, 1 << digit_bits, D) for _ in range(K)]
    tables = [gen.integers(0, 1 << out_bits, 1 << digit_bits) for _ in range(K)]
    Yk = [tables[k][X[k]] for k in range(K)]
    Y = np.ones(D, dtype=np.int64)
    for k in range(K):
        Y = Y * Yk[k]
    Zp = -sum(bases[k] * X[k] for k in range(K))
    yhat = [sum(int(v) for v in row) for row in Y.reshape(rows, cols)]  # may pass 2^63
    return Zp.astype(np.int64), X, Y, Yk, yhat, bases


def small_on_device(zk, orc, w):
    Zp, X, Y, Yk, yhat, bases = w
    i64 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int64)).cuda()
    u32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint32).view(np.int32)).cuda()
    yh = zk.vec_from_bytes(orc.to_bytes(yhat))
    return i64(Zp), [u32(a) for a in X], i64(Y), [u32(a) for a in Yk], yh, bases


def small_oracle_proof(orc, seed, w, rows, cols):
    Zp, X, Y, Yk, yhat, bases = w
    to = lambda a: orc.fr_from_i64(np.asarray(a, dtype=np.int64))
    return orc.zkattn_link_prove(seed, to(Zp), [to(a) for a in X], to(Y), [to(a) for a in Yk], orc.to_bytes(yhat),
                                 orc.to_bytes(bases), rows, cols)


@pytest.mark.parametrize("rows,cols,K,digit_bits,out_bits", [
    (2, 2, 2, 4, 8), (1, 4, 1, 8, 31), (4, 1, 2, 8, 16), (1, 1024, 2, 8, 16), (1024, 1, 2, 8, 16), (8, 512, 2, 16, 16),
    (64, 64, 1, 8, 20), (32, 128, 3, 5, 17), (512, 2, 3, 4, 9), (16, 4096, 2, 16, 29), (4, 16384, 2, 12, 16)])
def test_integer_tensors_give_the_same_proof(zk, orc, rows, cols, K, digit_bits, out_bits):
    gen = np.random.default_rng(rows * 131 + cols * 7 + K)
    w = small_witness(gen, rows, cols, K, digit_bits, out_bits)
    seed = bytes(gen.integers(0, 256, 32, dtype=np.uint8))
    rc_o, want, _ = small_oracle_proof(orc, seed, w, rows, cols)
    assert rc_o == 0
    Zp, X, Y, Yk, yhat, bases = small_on_device(zk, orc, w)
    rc, got = zk.zkattn_link_prove_small(seed, Zp, X, Y, Yk, yhat, bases, rows, cols)
    assert rc == zk.ZK_OK and got == want
    # the same bytes as from the tensors as field elements
    to = lambda a: zk.vec_from_bytes(orc.fr_from_i64(np.asarray(a, dtype=np.int64)))
    rc, again = zk.zkattn_link_prove(seed, to(w[0]), [to(a) for a in w[1]], to(w[2]), [to(a) for a in w[3]], yhat, bases,
                                     rows, cols)
    assert rc == zk.ZK_OK and again == got


def test_integer_tensors_extreme_values(zk, orc):
    """Entries at the ends of the ranges the integer path is written for: scores near
    -2^61 (a base of 2^32 - 1 against digits up to 2^29), segment outputs of 2^30 - 1
    against zero (the extrapolated factors change sign)."""
    rows, cols, K = 8, 64, 2
    D = rows * cols
    gen = np.random.default_rng(99)
    bases = [1, (1 << 32) - 1]
    X = [gen.integers(0, 1 << 32, D), gen.integers(0, 1 << 29, D)]
    Yk = [gen.choice([0, 1, (1 << 30) - 1], D), gen.choice([0, 1, (1 << 30) - 1], D)]
    Y = Yk[0] * Yk[1]
    Zp = -(X[0] + bases[1] * X[1])
    assert Zp.min() > -(1 << 62) and Y.max() < (1 << 62)
    yhat_int = [sum(int(v) for v in row) for row in Y.reshape(rows, cols)]
    w = (Zp, X, Y, Yk, None, bases)
    seed = b"\x42" * 32
    to = lambda a: orc.fr_from_i64(np.asarray(a, dtype=np.int64))
    rc_o, want, _ = orc.zkattn_link_prove(seed, to(Zp), [to(a) for a in X], to(Y), [to(a) for a in Yk],
                                          orc.to_bytes(yhat_int), orc.to_bytes(bases), rows, cols)
    assert rc_o == 0
    i64 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int64)).cuda()
    u32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint32).view(np.int32)).cuda()
    yh = zk.vec_from_bytes(orc.to_bytes(yhat_int))
    rc, got = zk.zkattn_link_prove_small(seed, i64(Zp), [u32(a) for a in X], i64(Y), [u32(a) for a in Yk], yh, bases,
                                         rows, cols)
    assert rc == zk.ZK_OK and got == want


def test_integer_tensors_refusals(zk, orc):
    gen = np.random.default_rng(7)
    rows, cols, K = 16, 256, 2
    w = small_witness(gen, rows, cols, K, 8, 16)
    seed = b"\x11" * 32
    Zp, X, Y, Yk, yhat, bases = small_on_device(zk, orc, w)
    assert zk.zkattn_link_prove_small(seed, Zp, X, Y, Yk, yhat, bases, rows, cols)[0] == zk.ZK_OK
    D = rows * cols

    def altered(t, pos, delta):
        c = t.clone()
        c[pos] += delta
        return c
    # each relation broken in one entry, anywhere in the tensor (both halves of the first round's pairs)
    for pos in (0, D // 2 - 1, D // 2, D - 1):
        assert zk.zkattn_link_prove_small(seed, altered(Zp, pos, 1), X, Y, Yk, yhat, bases, rows, cols)[0] == zk.ZK_E_REJECT
        assert zk.zkattn_link_prove_small(seed, Zp, [X[0], altered(X[1], pos, 1)], Y, Yk, yhat, bases, rows, cols)[0] == zk.ZK_E_REJECT
        assert zk.zkattn_link_prove_small(seed, Zp, X, altered(Y, pos, 1), Yk, yhat, bases, rows, cols)[0] == zk.ZK_E_REJECT
        assert zk.zkattn_link_prove_small(seed, Zp, X, Y, [altered(Yk[0], pos, 1), Yk[1]], yhat, bases, rows, cols)[0] == zk.ZK_E_REJECT
    # wrong row sums: seen where the first round's polynomial is compared with the claim
    bad_sums = list(w[4])
    bad_sums[3] += 1
    yh = zk.vec_from_bytes(orc.to_bytes(bad_sums))
    assert zk.zkattn_link_prove_small(seed, Zp, X, Y, Yk, yh, bases, rows, cols)[0] == zk.ZK_E_REJECT
    # out of range: a segment output of 2^30 with two segments, a score beyond 2^62
    big = Yk[0].clone()
    big[5] = 1 << 30
    assert zk.zkattn_link_prove_small(seed, Zp, X, Y, [big, Yk[1]], yhat, bases, rows, cols)[0] == zk.ZK_E_BADARG
    assert zk.zkattn_link_prove_small(seed, altered(Zp, 9, -(1 << 62)), X, Y, Yk, yhat, bases, rows, cols)[0] == zk.ZK_E_BADARG
    # arguments
    assert zk.zkattn_link_prove_small(seed, Zp, X, Y, Yk, yhat, [1, 0], rows, cols)[0] == zk.ZK_E_BADARG
    assert zk.zkattn_link_prove_small(seed, Zp, X, Y, Yk, yhat, [1, 1 << 32], rows, cols)[0] == zk.ZK_E_BADARG
    assert zk.zkattn_link_prove_small(seed, Zp, X, Y, Yk, yhat, bases, 1, 2)[0] == zk.ZK_E_BADARG   # fewer than four entries
    assert zk.zkattn_link_prove_small(seed, Zp, X, Y, Yk, yhat, bases, rows, cols, cap=10)[0] == zk.ZK_E_BUFSZ


def test_broken_relations_are_refused(zk, orc):
    rng = random.Random(21)
    rows, cols, K = 16, 256, 2
    w = make_witness(rng, rows, cols, K, digit_bits=8)
    seed = rng.randbytes(32)
    Zp, X, Y, Yk, yhat, bases = to_device(zk, orc, w)
    rc, proof = zk.zkattn_link_prove(seed, Zp, X, Y, Yk, yhat, bases, rows, cols)
    assert rc == zk.ZK_OK
    for which, sub in [(0, None), (1, 1), (2, None), (3, 0), (4, None)]:
        bad = [list(a) if not isinstance(a[0], list) else [list(b) for b in a] for a in w]
        target = bad[which] if sub is None else bad[which][sub]
        pos = rng.randrange(len(target))
        target[pos] = (target[pos] + 1) % R
        dZp, dX, dY, dYk, dyhat, _ = to_device(zk, orc, bad)
        assert zk.zkattn_link_prove(seed, dZp, dX, dY, dYk, dyhat, bases, rows, cols)[0] == zk.ZK_E_REJECT
        # the honest proof does not open to the altered tensors
        assert zk.zkattn_link_verify(seed, proof, rows, cols, bases, Zp=dZp, X=dX, Y=dY, Yk=dYk, yhat=dyhat)[0] == zk.ZK_E_REJECT
    assert zk.zkattn_link_verify(seed, proof, rows, cols, [1, 257])[0] == zk.ZK_E_REJECT


def test_argument_errors(zk, orc):
    rng = random.Random(22)
    w = make_witness(rng, 4, 4, 2)
    Zp, X, Y, Yk, yhat, bases = to_device(zk, orc, w)
    seed = b"\x07" * 32
    assert zk.zkattn_link_prove(seed, Zp, X, Y, Yk, yhat, bases, 3, 4)[0] == zk.ZK_E_BADARG
    assert zk.zkattn_link_prove(seed, Zp, X, Y, Yk, yhat, bases, 8, 4)[0] == zk.ZK_E_BADARG      # tensors too short
    assert zk.zkattn_link_prove(seed, Zp, X, Y, Yk, yhat, [1, 0], 4, 4)[0] == zk.ZK_E_BADARG     # a zero base
    assert zk.zkattn_link_prove(seed, Zp, X, Y, Yk, yhat, [1, R], 4, 4)[0] == zk.ZK_E_BADARG     # not canonical
    assert zk.zkattn_link_prove(seed, Zp, X, Y, Yk, yhat, bases, 4, 4, cap=10)[0] == zk.ZK_E_BUFSZ
