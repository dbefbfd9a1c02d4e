"""Pins of the oracle's product sumcheck and matmul proof (Section 6.1.1, with
the generic rounds of Section 3.3) against brute-force definitions and an
independently computed integer matrix product (no GPU)."""
import random

import numpy as np
import pytest

from tests import pyref
from tests.pyref import R


@pytest.mark.parametrize("d", [0, 1, 3, 5])
def test_product_proof_equals_definition(orc, d):
    rng = random.Random(40 + d)
    a = [rng.randrange(R) for _ in range(1 << d)]
    b = [rng.randrange(R) for _ in range(1 << d)]
    claim = sum(x * y for x, y in zip(a, b)) % R
    seed = rng.randbytes(32)
    expect, r = pyref.product_proof(seed, a, b, claim)
    rc, proof, rr = orc.sumcheck_prove_product(seed, orc.to_bytes(a), orc.to_bytes(b), orc.to_bytes([claim])[0], threads=3)
    assert rc == orc.OK and proof == expect and orc.to_ints(rr) == r
    assert orc.sumcheck_verify_product(seed, proof, 1 << d) == orc.OK
    assert orc.sumcheck_verify_product(seed, proof, 1 << d, a=orc.to_bytes(a), b=orc.to_bytes(b)) == orc.OK
    if d:
        for pos in rng.sample(range(len(proof)), 40):
            bad = bytearray(proof)
            bad[pos] ^= 1 << rng.randrange(8)
            assert orc.sumcheck_verify_product(seed, bytes(bad), 1 << d) == orc.E_REJECT, pos


def test_product_wrong_claim_is_rejected(orc):
    rng = random.Random(45)
    a = [rng.randrange(R) for _ in range(8)]
    b = [rng.randrange(R) for _ in range(8)]
    claim = (sum(x * y for x, y in zip(a, b)) + 1) % R
    rc, proof, _ = orc.sumcheck_prove_product(b"\x05" * 32, orc.to_bytes(a), orc.to_bytes(b), orc.to_bytes([claim])[0])
    assert rc == orc.OK
    assert orc.sumcheck_verify_product(b"\x05" * 32, proof, 8) == orc.E_REJECT


def test_matmul_two_by_two_by_hand(orc):
    # X = [[1,2],[3,4]], W = [[5,6],[7,8]], Y = [[19,22],[43,50]].
    # With u, v in F: Y~(u,v) = 19(1-u)(1-v) + 22(1-u)v + 43u(1-v) + 50uv,
    # a = (X~(u,0), X~(u,1)) = (1+2u, 2+2u), b = (W~(0,v), W~(1,v)) = (5+v, 7+v).
    seed = b"\x07" * 32
    X, W = np.array([[1, 2], [3, 4]]), np.array([[5, 6], [7, 8]])
    rc, proof, info = orc.matmul_sumcheck_prove(seed, X, W)
    assert rc == orc.OK
    u, v, r = (orc.to_ints(info[k])[0] for k in ("u", "v", "r"))
    claim = (19 * (1 - u) * (1 - v) + 22 * (1 - u) * v + 43 * u * (1 - v) + 50 * u * v) % R
    a0, a1, b0, b1 = 1 + 2 * u, 2 + 2 * u, 5 + v, 7 + v
    assert (a0 * b0 + a1 * b1) % R == claim
    el = [int.from_bytes(proof[32 + 32 * i:64 + 32 * i], "little") for i in range(6)]
    g = lambda x: (a0 + x * (a1 - a0)) * (b0 + x * (b1 - b0)) % R
    assert el == [claim, g(0), g(1), g(2), (a0 + r * (a1 - a0)) % R, (b0 + r * (b1 - b0)) % R]


@pytest.mark.parametrize("shape", [(1, 1, 1), (2, 3, 2), (4, 4, 4), (3, 5, 6), (8, 7, 2)])
def test_matmul_proof_equals_definition(orc, shape):
    D0, D1, D2 = shape
    rng = random.Random(50 + D0 * 100 + D1 * 10 + D2)
    X = [[rng.randrange(-300, 300) for _ in range(D1)] for _ in range(D0)]
    W = [[rng.randrange(-100, 100) for _ in range(D2)] for _ in range(D1)]
    seed = rng.randbytes(32)
    expect, ref = pyref.matmul_proof(seed, X, W)
    rc, proof, info = orc.matmul_sumcheck_prove(seed, np.array(X), np.array(W), threads=3)
    assert rc == orc.OK and proof == expect
    assert orc.to_ints(info["u"]) == ref["u"] and orc.to_ints(info["v"]) == ref["v"] and orc.to_ints(info["r"]) == ref["r"]
    # the claim is the MLE of an independent integer product (numpy int64)
    Y = np.array(X, dtype=np.int64) @ np.array(W, dtype=np.int64)
    assert Y.tolist() == ref["Y"]
    Yb = orc.fr_from_i64(Y.reshape(-1))
    assert orc.matmul_sumcheck_verify(seed, proof, D0, D1, D2, Y=Yb, X=np.array(X), W=np.array(W)) == orc.OK
    assert orc.matmul_sumcheck_verify(seed, proof, D0, D1, D2) == orc.OK
    Y2 = Y.copy()
    Y2[0, 0] += 1
    assert orc.matmul_sumcheck_verify(seed, proof, D0, D1, D2, Y=orc.fr_from_i64(Y2.reshape(-1))) == orc.E_REJECT
    X2 = np.array(X)
    X2[-1, -1] += 1
    assert orc.matmul_sumcheck_verify(seed, proof, D0, D1, D2, X=X2) == orc.E_REJECT
    if len(proof) > 160:
        bad = bytearray(proof)
        bad[100] ^= 4
        assert orc.matmul_sumcheck_verify(seed, bytes(bad), D0, D1, D2) == orc.E_REJECT
