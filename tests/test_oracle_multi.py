"""Pins of the oracle's tlookup over instances of unequal shapes (one sumcheck, all
claims at one point) against brute-force evaluation of the definitions (no GPU)."""
import random

import numpy as np
import pytest

from tests import pyref
from tests.pyref import R


def _instance(rng, D, N):
    T, seen = [], set()
    while len(T) < N:
        t = rng.randrange(R)
        if t not in seen:
            seen.add(t)
            T.append(t)
    return [rng.choice(T) for _ in range(D)], T


def _instances(rng, shapes):
    pairs = [_instance(rng, D, N) for D, N in shapes]
    return [p[0] for p in pairs], [p[1] for p in pairs]


SHAPES = [
    [(8, 2), (4, 4)],            # one variable apart
    [(4, 4), (8, 2)],            # the longer one second
    [(16, 4), (2, 1), (8, 8)],   # three shapes, three lengths
    [(1, 1), (8, 2)],            # an instance without variables
    [(32, 8), (4, 2)],           # three variables apart
    [(8, 4), (8, 2)],            # equal lengths, different tables
]


@pytest.mark.parametrize("shapes", SHAPES)
def test_multi_proof_equals_definition(orc, shapes):
    rng = random.Random(900 + sum(D * 31 + N for D, N in shapes))
    Ss, Ts = _instances(rng, shapes)
    seed = rng.randbytes(32)
    K = len(shapes)
    expect, ref = pyref.tlookup_multi_proof(seed, Ss, Ts)
    rc, proof, info = orc.tlookup_multi_prove(seed, [orc.to_bytes(s) for s in Ss], [orc.to_bytes(t) for t in Ts], threads=3)
    assert rc == orc.OK and proof == expect
    assert orc.to_ints(info["lambda"]) == [ref["lambda"]] and orc.to_ints(info["v"]) == ref["v"]
    # closed form of the honest claim: (sum_k lambda^k)(alpha + alpha^2), whatever the shapes
    lam_sum = sum(pow(ref["lambda"], k, R) for k in range(K)) % R
    g0 = ref["polys"][0]
    assert (g0[0] + g0[1]) % R == lam_sum * (ref["alpha"] + ref["alpha"] ** 2) % R
    assert np.array_equal(info["sum_A"], info["sum_mB"])
    Tb = [orc.to_bytes(t) for t in Ts]
    Ds = [D for D, _ in shapes]
    assert orc.tlookup_multi_verify(seed, proof, Tb, Ds) == orc.OK
    ms = [np.array(m, dtype=np.uint64) for m in ref["m"]]
    assert orc.tlookup_multi_verify(seed, proof, Tb, Ds, S_list=[orc.to_bytes(s) for s in Ss], m_list=ms) == orc.OK
    header = 16 + 16 * K
    for pos in rng.sample(range(len(proof)), min(60, len(proof))):
        # the digests of A and B of an instance without variables of its own bind nothing by themselves only if the
        # whole proof has no round; here there is always one, so every byte matters
        bad = bytearray(proof)
        bad[pos] ^= 1 << rng.randrange(8)
        assert orc.tlookup_multi_verify(seed, bytes(bad), Tb, Ds) == orc.E_REJECT, (pos, header)


def test_equal_shapes_frame_like_the_batched_proof(orc):
    # With all shapes equal f is the batched proof's f (both provers are pinned to the brute force, which builds the two
    # from the same terms); the transcripts differ by label and header, so only the framing can be compared here.
    rng = random.Random(5)
    Ss, Ts = _instances(rng, [(16, 4), (16, 4)])
    seed = rng.randbytes(32)
    Sb, Tb = [orc.to_bytes(s) for s in Ss], [orc.to_bytes(t) for t in Ts]
    rc1, p1, i1 = orc.tlookup_multi_prove(seed, Sb, Tb)
    rc2, p2, i2 = orc.tlookup_batch_prove(seed, Sb, Tb)
    assert rc1 == orc.OK and rc2 == orc.OK
    assert len(p1) == len(p2) + 16  # K, K x (D, N) instead of D, N, K
    assert p1[:4] == b"ZKTM" and p2[:4] == b"ZKTB"
    # the digests of m do not depend on the transcript
    assert p1[16 + 32:16 + 32 + 64] == p2[32:32 + 64]


def test_multi_rejects_bad_shapes_and_missing_rows(orc):
    rng = random.Random(11)
    Ss, Ts = _instances(rng, [(8, 2), (4, 4)])
    seed = rng.randbytes(32)
    Sb, Tb = [orc.to_bytes(s) for s in Ss], [orc.to_bytes(t) for t in Ts]
    # an entry that is in no row of its table
    bad = [list(s) for s in Ss]
    bad[1][2] = (max(Ts[1]) + 1) % R
    while bad[1][2] in Ts[1]:
        bad[1][2] = (bad[1][2] + 1) % R
    rc, _, info = orc.tlookup_multi_prove(seed, [orc.to_bytes(s) for s in bad], Tb)
    assert rc == orc.E_NOT_IN_TABLE and info["bad_instance"] == 1 and info["bad_index"] == 2
    # lengths that are not powers of two, or a table longer than its tensor
    rc, _, _ = orc.tlookup_multi_prove(seed, [Sb[0][:6], Sb[1]], Tb)
    assert rc == orc.E_BADARG
    rc, _, _ = orc.tlookup_multi_prove(seed, [Sb[0][:1], Sb[1]], Tb)
    assert rc == orc.E_BADARG
    # a proof is bound to the order and the shapes of its instances
    rc, proof, _ = orc.tlookup_multi_prove(seed, Sb, Tb)
    assert rc == orc.OK
    assert orc.tlookup_multi_verify(seed, proof, Tb[::-1], [4, 8]) == orc.E_REJECT
    assert orc.tlookup_multi_verify(seed, proof, Tb, [8, 4]) == orc.OK
