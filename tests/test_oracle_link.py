"""Pins of the oracle's zkAttn linking sumcheck (oracle/zkattn_link.hpp; Protocol 2,
last step, with the relations of Section 5.1) against the definitions written out
in Python integers (tests/pyref.py), the closed form of the claim, round
consistency, the degree bound, and the verifier's behaviour on bad witnesses and
corrupted proofs."""
import random

import numpy as np
import pytest

from tests import pyref
from tests.pyref import R


def make_witness(rng, rows, cols, K, digit_bits=4, small_tables=True):
    """A witness that satisfies the three relations: digits of -Z', table outputs
    from arbitrary per-segment tables, their product and its row sums."""
    D = rows * cols
    base = 1 << digit_bits
    bases = [base ** k for k in range(K)]
    tables = [[rng.randrange(1, 50 if small_tables else R) for _ in range(base)] for _ in range(K)]
    X = [[rng.randrange(base) for _ in range(D)] for _ in range(K)]
    Zp = [(-sum(bases[k] * X[k][i] for k in range(K))) % R for i in range(D)]
    Yk = [[tables[k][X[k][i]] for i in range(D)] for k in range(K)]
    Y = [1] * D
    for k in range(K):
        Y = [Y[i] * Yk[k][i] % R for i in range(D)]
    yhat = [sum(Y[r * cols:(r + 1) * cols]) % R for r in range(rows)]
    return Zp, X, Y, Yk, yhat, bases


def prove(orc, seed, w, rows, cols):
    Zp, X, Y, Yk, yhat, bases = w
    return orc.zkattn_link_prove(seed, orc.to_bytes(Zp), [orc.to_bytes(a) for a in X], orc.to_bytes(Y),
                                 [orc.to_bytes(a) for a in Yk], orc.to_bytes(yhat), orc.to_bytes(bases), rows, cols)


@pytest.mark.parametrize("rows,cols,K", [(2, 4, 2), (4, 2, 1), (1, 8, 2), (8, 1, 2), (2, 2, 3), (4, 4, 2)])
def test_proof_equals_the_definitions(orc, rows, cols, K):
    rng = random.Random(rows * 100 + cols * 10 + K)
    w = make_witness(rng, rows, cols, K, small_tables=False)
    seed = rng.randbytes(32)
    rc, proof, point = prove(orc, seed, w, rows, cols)
    assert rc == 0
    want, info = pyref.zkattn_link_proof(seed, *w, rows, cols)
    assert proof == want
    assert orc.to_ints(point) == info["v"]
    n = (rows * cols).bit_length() - 1
    # the claim's closed form, round consistency, and the degree bound K + 1
    claim = info["alpha"] ** 2 * info["cy"] % R
    assert sum(info["f"](pyref.bits_msb_first(x, n)) for x in range(rows * cols)) % R == claim
    for k, g in enumerate(info["polys"]):
        assert (g[0] + g[1]) % R == claim
        diffs = list(g)
        for _ in range(K + 2):
            diffs = [(b - a) % R for a, b in zip(diffs, diffs[1:])]
        assert all(d == 0 for d in diffs)          # (K+2)-th finite difference of a degree K+1 polynomial
        claim = int.from_bytes(orc.lagrange_eval(orc.to_bytes(g[:K + 2]), orc.to_bytes([info["v"][k]])[0]).tobytes(), "little")
    assert claim == info["f"](info["v"])
    assert orc.zkattn_link_verify(seed, proof, rows, cols, orc.to_bytes(w[5])) == 0


def test_single_entry(orc):
    rng = random.Random(3)
    w = make_witness(rng, 1, 1, 2)
    seed = b"\x05" * 32
    rc, proof, _ = prove(orc, seed, w, 1, 1)
    assert rc == 0 and proof == pyref.zkattn_link_proof(seed, *w, 1, 1)[0]
    assert orc.zkattn_link_verify(seed, proof, 1, 1, orc.to_bytes(w[5])) == 0
    bad = [list(a) if not isinstance(a[0], list) else [list(b) for b in a] for a in w]
    bad[2][0] = (bad[2][0] + 1) % R
    assert prove(orc, seed, bad, 1, 1)[0] == orc.E_REJECT


def test_each_relation_is_enforced(orc):
    """Breaking any one of the three relations at a single entry makes the prover's
    own first-round check fail; a proof for the honest witness does not verify
    against the altered tensors."""
    rng = random.Random(11)
    rows, cols, K = 4, 8, 2
    w = make_witness(rng, rows, cols, K)
    seed = rng.randbytes(32)
    rc, proof, _ = prove(orc, seed, w, rows, cols)
    assert rc == 0
    to = orc.to_bytes
    full = dict(Zp=to(w[0]), X_list=[to(a) for a in w[1]], Y=to(w[2]), Yk_list=[to(a) for a in w[3]], yhat=to(w[4]))
    assert orc.zkattn_link_verify(seed, proof, rows, cols, to(w[5]), **full) == 0

    def altered(which, sub=None):
        c = [list(a) if not isinstance(a[0], list) else [list(b) for b in a] for a in w]
        pos = rng.randrange(len(c[which]) if sub is None else len(c[which][sub]))
        if sub is None:
            c[which][pos] = (c[which][pos] + 1) % R
        else:
            c[which][sub][pos] = (c[which][sub][pos] + 1) % R
        return c

    for which, sub in [(0, None), (1, 0), (1, 1), (2, None), (3, 0), (3, 1), (4, None)]:
        bad = altered(which, sub)
        assert prove(orc, seed, bad, rows, cols)[0] == orc.E_REJECT, (which, sub)
        args = dict(Zp=to(bad[0]), X_list=[to(a) for a in bad[1]], Y=to(bad[2]), Yk_list=[to(a) for a in bad[3]],
                    yhat=to(bad[4]))
        assert orc.zkattn_link_verify(seed, proof, rows, cols, to(w[5]), **args) == orc.E_REJECT, (which, sub)
    # a different base is a different statement
    assert orc.zkattn_link_verify(seed, proof, rows, cols, to([1, 17])) == orc.E_REJECT


def test_corrupted_proofs_are_rejected(orc):
    rng = random.Random(12)
    rows, cols, K = 2, 8, 2
    w = make_witness(rng, rows, cols, K)
    seed = rng.randbytes(32)
    rc, proof, _ = prove(orc, seed, w, rows, cols)
    assert rc == 0 and len(proof) == 64 + 4 * (K + 2) * 32 + (2 * K + 2) * 32
    bases = orc.to_bytes(w[5])
    for pos in rng.sample(range(len(proof)), 60):
        bad = bytearray(proof)
        bad[pos] ^= 1 << rng.randrange(8)
        assert orc.zkattn_link_verify(seed, bytes(bad), rows, cols, bases) == orc.E_REJECT, pos
    assert orc.zkattn_link_verify(seed, proof[:-1], rows, cols, bases) == orc.E_REJECT
    assert orc.zkattn_link_verify(b"\x00" * 32, proof, rows, cols, bases) == orc.E_REJECT
    assert orc.zkattn_link_verify(seed, proof, cols, rows, bases) == orc.E_REJECT
    assert orc.zkattn_link_verify(seed, proof, 3, cols, bases) == orc.E_BADARG


def test_larger_instance_is_self_consistent(orc):
    """At a size brute force cannot reach: prove, verify with every tensor given."""
    rng = random.Random(13)
    rows, cols, K = 16, 64, 2
    w = make_witness(rng, rows, cols, K, digit_bits=8)
    seed = rng.randbytes(32)
    rc, proof, _ = prove(orc, seed, w, rows, cols)
    assert rc == 0
    to = orc.to_bytes
    assert orc.zkattn_link_verify(seed, proof, rows, cols, to(w[5]), Zp=to(w[0]), X_list=[to(a) for a in w[1]], Y=to(w[2]),
                                  Yk_list=[to(a) for a in w[3]], yhat=to(w[4])) == 0
