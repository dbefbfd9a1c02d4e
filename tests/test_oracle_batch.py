"""Pins of the oracle's batched tlookup (several instances under one sumcheck)
against brute-force evaluation of the definitions (no GPU)."""
import random

import numpy as np
import pytest

from tests import pyref
from tests.pyref import R


def _instances(rng, K, D, N):
    Ss, Ts = [], []
    for _ in range(K):
        T, seen = [], set()
        while len(T) < N:
            t = rng.randrange(R)
            if t not in seen:
                seen.add(t)
                T.append(t)
        Ts.append(T)
        Ss.append([rng.choice(T) for _ in range(D)])
    return Ss, Ts


@pytest.mark.parametrize("K,D,N", [(1, 8, 2), (2, 1, 1), (2, 4, 4), (2, 16, 4), (3, 8, 1), (2, 32, 8)])
def test_batch_proof_equals_definition(orc, K, D, N):
    rng = random.Random(500 + 100 * K + D + N)
    Ss, Ts = _instances(rng, K, D, N)
    seed = rng.randbytes(32)
    expect, ref = pyref.tlookup_batch_proof(seed, Ss, Ts)
    rc, proof, info = orc.tlookup_batch_prove(seed, [orc.to_bytes(s) for s in Ss], [orc.to_bytes(t) for t in Ts], threads=3)
    assert rc == orc.OK and proof == expect
    assert orc.to_ints(info["lambda"]) == [ref["lambda"]] and orc.to_ints(info["v"]) == ref["v"]
    # closed form of the honest claim: (sum_k lambda^k)(alpha + alpha^2)
    if D > 1:
        lam_sum = sum(pow(ref["lambda"], k, R) for k in range(K)) % R
        assert ref["first_claim"] == lam_sum * (ref["alpha"] + ref["alpha"] ** 2) % R
    # log-derivative identity per instance
    assert np.array_equal(info["sum_A"], info["sum_mB"])
    Tb = [orc.to_bytes(t) for t in Ts]
    assert orc.tlookup_batch_verify(seed, proof, Tb, D) == orc.OK
    ms = [np.array(m, dtype=np.uint64) for m in ref["m"]]
    assert orc.tlookup_batch_verify(seed, proof, Tb, D, S_list=[orc.to_bytes(s) for s in Ss], m_list=ms) == orc.OK
    for pos in rng.sample(range(len(proof)), min(40, len(proof))):
        # With D = 1 there is no round and the honest final claims satisfy the last identity for every
        # alpha and lambda, so the digests of A and B (which only feed those challenges) bind nothing.
        if D == 1 and 32 + 32 * K <= pos < 32 + 96 * K:
            continue
        bad = bytearray(proof)
        bad[pos] ^= 1 << rng.randrange(8)
        assert orc.tlookup_batch_verify(seed, bytes(bad), Tb, D) == orc.E_REJECT, pos


def test_single_instance_batch_differs_only_by_framing(orc):
    # K = 1: same sums as the plain prover under a different transcript label
    rng = random.Random(9)
    Ss, Ts = _instances(rng, 1, 16, 4)
    seed = rng.randbytes(32)
    rc, proof, _ = orc.tlookup_batch_prove(seed, [orc.to_bytes(Ss[0])], [orc.to_bytes(Ts[0])])
    assert rc == orc.OK and proof[:4] == b"ZKTB" and len(proof) == 32 + 96 + 4 * 128 + 160


def test_batch_errors(orc):
    rng = random.Random(10)
    Ss, Ts = _instances(rng, 2, 16, 4)
    Sb = [orc.to_bytes(s) for s in Ss]
    Tb = [orc.to_bytes(t) for t in Ts]
    Sb[1] = Sb[1].copy()
    Sb[1][5] = orc.to_bytes([12345])[0]
    rc, _, info = orc.tlookup_batch_prove(b"\x00" * 32, Sb, Tb)
    assert rc == orc.E_NOT_IN_TABLE and info["bad_instance"] == 1 and info["bad_index"] == 5
