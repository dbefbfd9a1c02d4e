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
