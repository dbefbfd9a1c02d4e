"""Pins of the oracle's tlookup prover/verifier (Section 4, Protocol 1) against
the definitions evaluated by brute force, the closed forms of the honest claim
and library counting (no GPU)."""
import random

import numpy as np
import pytest

from tests import pyref
from tests.pyref import R


def _instance(rng, D, N, table=None, dup=False):
    T = table
    if T is None:
        T = []
        while len(T) < N:
            t = rng.randrange(R)
            if t not in T:
                T.append(t)
    if dup and N >= 4:
        T[N - 1] = T[1]
    S = [rng.choice(T) for _ in range(D)]
    return S, T


def test_multiplicities_match_bincount_and_sum_to_D(orc):
    rng = np.random.default_rng(5)
    N, D = 64, 4096
    idx = rng.integers(0, N, D)
    T = orc.fr_from_i64(np.arange(-32, 32))
    S = T[idx]
    rc, m, _ = orc.multiplicities(S, T, threads=3)
    assert rc == orc.OK
    assert np.array_equal(m, np.bincount(idx, minlength=N).astype(np.uint64))
    assert int(m.sum()) == D


def test_multiplicities_duplicates_go_to_lowest_row(orc):
    T = orc.to_bytes([5, 9, 5, 7])
    S = orc.to_bytes([5, 5, 7, 9, 5, 7, 7, 7])
    rc, m, _ = orc.multiplicities(S, T)
    assert rc == orc.OK and list(m) == [3, 1, 0, 4]


def test_not_in_table_reports_smallest_index(orc):
    T = orc.to_bytes([1, 2, 3, 4])
    S = orc.to_bytes([1, 2, 9, 4, 8, 1, 1, 1])
    rc, _, bad = orc.multiplicities(S, T, threads=4)
    assert rc == orc.E_NOT_IN_TABLE and bad == 2
    rc, proof, info = orc.tlookup_prove(b"\x01" * 32, S, T)
    assert rc == orc.E_NOT_IN_TABLE and info["bad_index"] == 2


def test_m_digest_against_hashlib(orc):
    rng = np.random.default_rng(6)
    for N in (1, 4, 128, 129, 1024):
        m = rng.integers(0, 2 ** 31, N).astype(np.uint64)
        assert orc.m_digest(m) == pyref.m_digest([int(c) for c in m])


def test_vec_digest_against_hashlib(orc):
    """The stand-in for the commitments of A and B: strided leaves of 128 elements,
    then rows of digests hashed in fours (a last pair in twos)."""
    import hashlib
    rng = random.Random(7)
    for n in (1, 2, 4, 64, 128, 256, 512, 1024, 2048, 4096, 8192, 1 << 15):
        vals = [rng.randrange(R) for _ in range(n)]
        assert orc.vec_digest(orc.to_bytes(vals), threads=3) == pyref.vec_digest(vals), n
    # the shape of the tree, spelled out once for n = 512: four leaves, element x in leaf x mod 4
    vals = [rng.randrange(R) for _ in range(512)]
    leaves = [hashlib.sha256(b"".join(pyref.fr_bytes(vals[x]) for x in range(i, 512, 4))).digest() for i in range(4)]
    assert orc.vec_digest(orc.to_bytes(vals)) == hashlib.sha256(b"".join(leaves)).digest()
    # n = 256: two leaves, hashed as a pair
    leaves = [hashlib.sha256(b"".join(pyref.fr_bytes(vals[x]) for x in range(i, 256, 2))).digest() for i in range(2)]
    assert orc.vec_digest(orc.to_bytes(vals[:256])) == hashlib.sha256(leaves[0] + leaves[1]).digest()
    # below one leaf: the hash of the elements in order
    assert orc.vec_digest(orc.to_bytes(vals[:8])) == hashlib.sha256(b"".join(pyref.fr_bytes(x) for x in vals[:8])).digest()


def test_inverse_vectors_are_sent_before_the_sumcheck(orc):
    """Protocol 1: A and B go to the verifier after beta and before the sumcheck, so
    alpha and u must depend on them and beta must not.  The proof carries their
    digests after that of m; alpha is recomputed here from the transcript rules."""
    rng = random.Random(36)
    D, N = 32, 8
    S, T = _instance(rng, D, N)
    seed = rng.randbytes(32)
    rc, proof, info = orc.tlookup_prove(seed, orc.to_bytes(S), orc.to_bytes(T))
    assert rc == orc.OK and proof[:8] == b"ZKTL" + (2).to_bytes(4, "little")
    beta = orc.to_ints(info["beta"])[0]
    A = [pow(beta + s, -1, R) for s in S]
    B = [pow(beta + t, -1, R) for t in T]
    assert proof[56:88] == pyref.vec_digest(A) and proof[88:120] == pyref.vec_digest(B)
    tr = pyref.Transcript(b"zkmi/tlookup/v2" + seed + D.to_bytes(8, "little") + N.to_bytes(8, "little"))
    tr.absorb("m", proof[24:56])
    assert tr.challenge("beta") == beta
    tr.absorb("A", proof[56:88])
    tr.absorb("B", proof[88:120])
    assert tr.challenge("alpha") == orc.to_ints(info["alpha"])[0]
    assert [tr.challenge("u") for _ in range(5)] == orc.to_ints(info["u"])


@pytest.mark.parametrize("D,N,dup", [(1, 1, False), (2, 1, False), (8, 1, False), (4, 4, False), (8, 8, True),
                                     (16, 4, False), (16, 2, False), (32, 8, True)])
def test_proof_equals_brute_force_definition(orc, D, N, dup):
    rng = random.Random(100 + D * 7 + N)
    S, T = _instance(rng, D, N, dup=dup)
    seed = rng.randbytes(32)
    expect, ref = pyref.tlookup_proof(seed, S, T)
    rc, proof, info = orc.tlookup_prove(seed, orc.to_bytes(S), orc.to_bytes(T), threads=3)
    assert rc == orc.OK
    assert proof == expect
    assert orc.to_ints(info["beta"]) == [ref["beta"]] and orc.to_ints(info["alpha"]) == [ref["alpha"]]
    assert orc.to_ints(info["u"]) == ref["u"] and orc.to_ints(info["v"]) == ref["v"]
    # degree <= 3: the value at X = 4 from the definition equals the cubic through the four sent values
    n = D.bit_length() - 1
    for k in range(n):
        sent = orc.to_bytes(ref["polys"][k][:4])
        assert orc.to_ints(orc.lagrange_eval(sent, orc.to_bytes([4])[0])) == [ref["polys"][k][4]]


def test_honest_claim_closed_forms(orc):
    rng = random.Random(31)
    D, N = 64, 8
    S, T = _instance(rng, D, N)
    seed = rng.randbytes(32)
    rc, proof, info = orc.tlookup_prove(seed, orc.to_bytes(S), orc.to_bytes(T))
    assert rc == orc.OK
    beta, alpha = orc.to_ints(info["beta"])[0], orc.to_ints(info["alpha"])[0]
    # log-derivative identity at beta (Section 4, Lemma and the check after it)
    assert np.array_equal(info["sum_A"], info["sum_mB"])
    assert orc.to_ints(info["sum_A"])[0] == sum(pow(beta + s, -1, R) for s in S) % R
    # g_0(0) + g_0(1) = alpha + alpha^2
    g0 = [int.from_bytes(proof[120 + 32 * i:152 + 32 * i], "little") for i in range(2)]
    assert sum(g0) % R == (alpha + alpha * alpha) % R


def test_round_consistency_and_final_identity(orc):
    rng = random.Random(32)
    D, N = 128, 16
    S, T = _instance(rng, D, N)
    seed = rng.randbytes(32)
    Sb, Tb = orc.to_bytes(S), orc.to_bytes(T)
    rc, proof, info = orc.tlookup_prove(seed, Sb, Tb)
    assert rc == orc.OK
    n, h = 7, 3
    beta, alpha = orc.to_ints(info["beta"])[0], orc.to_ints(info["alpha"])[0]
    el = [int.from_bytes(proof[120 + 32 * i:152 + 32 * i], "little") for i in range(4 * n + 5)]
    v, u = orc.to_ints(info["v"]), orc.to_ints(info["u"])
    claim = (alpha + alpha * alpha) % R
    for k in range(n):
        g = el[4 * k:4 * k + 4]
        assert (g[0] + g[1]) % R == claim
        claim = orc.to_ints(orc.lagrange_eval(orc.to_bytes(g), orc.to_bytes([v[k]])[0]))[0]
    Av, Sv, Bv, mv, Tv = el[4 * n:]
    # final claims are the brute-force MLE values
    m = [sum(1 for s in S if s == t) for t in T]
    A = [pow(beta + s, -1, R) for s in S]
    B = [pow(beta + t, -1, R) for t in T]
    assert [Av, Sv, Bv, mv, Tv] == [pyref.mle(A, v), pyref.mle(S, v), pyref.mle(B, v[h:]), pyref.mle(m, v[h:]),
                                    pyref.mle(T, v[h:])]
    scale = pow(2 ** h, -1, R)
    rhs = Av * (alpha * pyref.eq(u, v) % R * (Sv + beta) + 1) + scale * Bv * (alpha * alpha % R * pyref.eq(u[h:], v[h:]) % R * (Tv + beta) - mv)
    assert rhs % R == claim


def test_verify_accepts_and_rejects(orc):
    rng = random.Random(33)
    D, N = 64, 16
    S, T = _instance(rng, D, N)
    seed = rng.randbytes(32)
    Sb, Tb = orc.to_bytes(S), orc.to_bytes(T)
    rc, proof, info = orc.tlookup_prove(seed, Sb, Tb)
    assert rc == orc.OK
    rcm, m, _ = orc.multiplicities(Sb, Tb)
    beta = info["beta"]
    _, A = orc.fr_inv(orc.fr_axpy(Sb, beta))
    _, B = orc.fr_inv(orc.fr_axpy(Tb, beta))
    rc, out = orc.tlookup_verify(seed, proof, Tb, D)
    assert rc == orc.OK and out["stage"] == 0
    assert np.array_equal(out["v"], info["v"])
    rc, out = orc.tlookup_verify(seed, proof, Tb, D, S=Sb, m=m, A=A, B=B)
    assert rc == orc.OK
    # any single corrupted byte is rejected
    for pos in list(range(0, 120)) + rng.sample(range(120, len(proof)), 60):
        bad = bytearray(proof)
        bad[pos] ^= 1 << rng.randrange(8)
        rc, out = orc.tlookup_verify(seed, bytes(bad), Tb, D)
        assert rc == orc.E_REJECT, pos
    # wrong seed, wrong witness, truncated proof
    assert orc.tlookup_verify(b"\x00" * 32, proof, Tb, D)[0] == orc.E_REJECT
    assert orc.tlookup_verify(seed, proof[:-1], Tb, D)[0] == orc.E_REJECT
    m2 = m.copy()
    m2[0] += 1
    assert orc.tlookup_verify(seed, proof, Tb, D, m=m2)[0] == orc.E_REJECT
    S2 = Sb.copy()
    S2[3] = Tb[1] if np.array_equal(Sb[3], Tb[0]) else Tb[0]
    assert orc.tlookup_verify(seed, proof, Tb, D, S=S2)[0] == orc.E_REJECT
    # inverse vectors other than the ones whose digests were sent
    A2 = A.copy()
    A2[[0, 1]] = A2[[1, 0]]
    assert not np.array_equal(A2[0], A[0])
    assert orc.tlookup_verify(seed, proof, Tb, D, A=A2)[0] == orc.E_REJECT
    B2 = B.copy()
    B2[[0, 1]] = B2[[1, 0]]
    assert orc.tlookup_verify(seed, proof, Tb, D, B=B2)[0] == orc.E_REJECT


def test_zero_denominator_is_reported(orc):
    rng = random.Random(34)
    S, T = _instance(rng, 16, 4)
    Sb, Tb = orc.to_bytes(S), orc.to_bytes(T)
    forced = orc.to_bytes([(-S[5]) % R])[0]
    rc, _, _ = orc.tlookup_prove(b"\x02" * 32, Sb, Tb, forced_beta=forced)
    assert rc == orc.E_ZERO_DENOM
    unused = [t for t in T if t not in S]
    if unused:
        forced = orc.to_bytes([(-unused[0]) % R])[0]
        assert orc.tlookup_prove(b"\x02" * 32, Sb, Tb, forced_beta=forced)[0] == orc.E_ZERO_DENOM


def test_bad_shapes(orc):
    T = orc.to_bytes([1, 2, 3])
    S = orc.to_bytes([1, 2, 3, 1])
    assert orc.tlookup_prove(b"\x00" * 32, S, T)[0] == orc.E_BADARG          # N not a power of two
    T = orc.to_bytes(list(range(8)))
    assert orc.tlookup_prove(b"\x00" * 32, S, T)[0] == orc.E_BADARG          # N > D
    S = orc.to_bytes([1, 2, 3, 1, 2, 3])
    assert orc.tlookup_prove(b"\x00" * 32, S, orc.to_bytes([1, 2]))[0] == orc.E_BADARG
    S, T = orc.to_bytes([1, 2, 1, 2]), orc.to_bytes([1, 2])
    rc, _, info = orc.tlookup_prove(b"\x00" * 32, S, T, cap=10)
    assert rc == orc.E_BUFSZ and info["len"] == orc.tlookup_proof_bytes(4)


def test_thread_count_does_not_change_bytes(orc):
    rng = random.Random(35)
    S, T = _instance(rng, 256, 16)
    seed = rng.randbytes(32)
    Sb, Tb = orc.to_bytes(S), orc.to_bytes(T)
    p1 = orc.tlookup_prove(seed, Sb, Tb, threads=1)[1]
    p5 = orc.tlookup_prove(seed, Sb, Tb, threads=5)[1]
    assert p1 == p5 and len(p1) == 280 + 128 * 8
