"""The rounds of a tlookup proof that the prover leaves to the host (at most 32
pairs: the resident kernel hands the five arrays over and the host computes the
sums, folds and final claims), checked here without a GPU against the sums'
definitions written out on Python integers: Section 3.3's sumcheck round over
the pairs (p, p + half), Section 4's summand split into the kernels' eleven sums,
weights e~(u_rest, p) with the first coordinate on the top bit of p."""
import random

import pytest

R = 0x73eda753299d7d483339d80809a1d80553bda402fffe5bfeffffffff00000001


def _eq(u, p, bits):
    """e~(u, p): product over the bits of p, u[0] on the top one."""
    w = 1
    for t in range(bits):
        b = (p >> (bits - 1 - t)) & 1
        w = w * (u[t] if b else (1 - u[t])) % R
    return w


def _expected(A, S, B, M, T, u_rest, beta, challenges):
    A, S, B, M, T = list(A), list(S), list(B), list(M), list(T)
    sums, k = [], 0
    half = len(A) // 2
    while half >= 1:
        bits = half.bit_length() - 1
        u = u_rest[len(u_rest) - bits:]  # the coordinates of the variables still free after this round's
        table = 2 * half <= len(B)
        out = [0] * 11
        for p in range(half):
            w = _eq(u, p, bits)
            out[0] += w * A[p] * (S[p] + beta)
            out[1] += w * A[p + half] * (S[p + half] + beta)
            out[2] += w * (A[p + half] - A[p]) * (S[p + half] - S[p])
            out[3] += A[p]
            out[4] += A[p + half]
            if table:
                out[5] += w * B[p] * (T[p] + beta)
                out[6] += w * B[p + half] * (T[p + half] + beta)
                out[7] += w * (B[p + half] - B[p]) * (T[p + half] - T[p])
                out[8] += B[p] * M[p]
                out[9] += B[p + half] * M[p + half]
                out[10] += (B[p + half] - B[p]) * (M[p + half] - M[p])
        sums += [x % R for x in out]
        r = challenges[k]
        fold = lambda x: [(x[p] + r * (x[p + half] - x[p])) % R for p in range(half)]
        A, S = fold(A), fold(S)
        if table:
            B, M, T = fold(B), fold(M), fold(T)
        half //= 2
        k += 1
    return sums, [A[0], S[0], B[0], M[0], T[0]]


@pytest.mark.parametrize("n_data,n_table", [(64, 64), (64, 16), (64, 1), (32, 32), (16, 2), (8, 8), (4, 1), (2, 2), (2, 1)])
def test_host_rounds_against_the_definition(n_data, n_table):
    import paper_2404_16109_amd as zk
    rng = random.Random(1000 * n_data + n_table)
    rnd = lambda n: [rng.randrange(R) for _ in range(n)]
    A, S, B, M, T = rnd(n_data), rnd(n_data), rnd(n_table), rnd(n_table), rnd(n_table)
    d = n_data.bit_length() - 1
    u_rest, beta, challenges = rnd(d - 1), rng.randrange(R), rnd(d)
    rc, sums, finals = zk.zkmi_selftest_host_rounds(A, S, B, M, T, u_rest, beta, challenges)
    assert rc == d
    want_sums, want_finals = _expected(A, S, B, M, T, u_rest, beta, challenges)
    assert sums == want_sums
    assert finals == want_finals


def test_host_rounds_extreme_values_and_degenerate_challenges():
    import paper_2404_16109_amd as zk
    n = 64
    A, S = [R - 1] * n, [R - 1 - (i % 3) for i in range(n)]
    B, M, T = [R - 1] * n, [0, R - 1] * (n // 2), [R - 2] * n
    u_rest, beta = [0, 1, R - 1, 1, 0], R - 1
    challenges = [0, 1, R - 1, 2, 0, 1]
    rc, sums, finals = zk.zkmi_selftest_host_rounds(A, S, B, M, T, u_rest, beta, challenges)
    assert rc == 6
    want_sums, want_finals = _expected(A, S, B, M, T, u_rest, beta, challenges)
    assert sums == want_sums and finals == want_finals


def test_host_rounds_argument_errors():
    import paper_2404_16109_amd as zk
    ok = [1] * 4
    assert zk.zkmi_selftest_host_rounds([1] * 3, [1] * 3, [1], [1], [1], [1], 1, [1, 1])[0] == zk.ZK_E_BADARG     # not a power of two
    assert zk.zkmi_selftest_host_rounds([1] * 128, [1] * 128, [1], [1], [1], [1] * 6, 1, [1] * 7)[0] == zk.ZK_E_BADARG  # too long
    assert zk.zkmi_selftest_host_rounds(ok, ok, [1] * 8, [1] * 8, [1] * 8, [1], 1, [1, 1])[0] == zk.ZK_E_BADARG   # table longer than data
    assert zk.zkmi_selftest_host_rounds(ok, ok, [1], [1], [1], [R], 1, [1, 1])[0] == zk.ZK_E_BADARG                # not canonical
