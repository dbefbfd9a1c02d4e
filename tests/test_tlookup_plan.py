"""The per-round plan of the tlookup prover (which kernel runs a round, where it
reads S from), walked on the host without a GPU through the same function the
prover uses.  What is pinned here is what a kernel launch relies on: a round
never has a source of S the library has no kernel for, integers are read only by
the two kernels written for them, and a round reads the layout the round before
it has written.  From a vector of field elements the first pass may serve the
first two rounds (FIRST_TWO, then NO_PASS: nothing launched), after which the
29-bit kernel binds two variables at once from the caller's arrays.  The last
rounds of a single proof (at most 32 pairs, once the resident kernel has run) are
the host's (HOST)."""
import pytest

FIRST, R29, BOTH, ONE_GROUP, RESIDENT, FIRST_TWO, NO_PASS, HOST = 0, 1, 2, 3, 4, 5, 6, 7
CALLER, INTS, WORDS, PLANES = 0, 1, 2, 3


def _plan(zk, D, N, K=1, from_ints=False):
    rc, rounds = zk.zkmi_selftest_tlookup_plan(D, N, K, from_ints)
    return rc, rounds


def _check_chain(rounds):
    """Round k >= 2 reads what round k-1 wrote: 29-bit planes after a 29-bit round that
    did not write words, 32-bit words otherwise; a 29-bit round that reads planes has
    in32 = 0."""
    shared = len(rounds) > 0 and rounds[0][0] == FIRST_TWO
    if shared:
        # one pass for two rounds, then both variables bound at once from the arrays as the caller left them
        assert len(rounds) >= 3 and rounds[1][0] == NO_PASS and rounds[2][0] == R29
        assert [r[1] for r in rounds[:3]] == [CALLER] * 3 and rounds[2][2] == 1
    assert all(r[0] not in (FIRST_TWO, NO_PASS) for r in rounds[2:]) and (shared or all(r[0] != NO_PASS for r in rounds))
    for k, (kernel, src, in32, out32) in enumerate(rounds):
        assert src in (CALLER, INTS, WORDS, PLANES), (k, src)
        if k <= 1 or (shared and k == 2):
            assert src in (CALLER, INTS)
            continue
        pk, _, _, pout32 = rounds[k - 1]
        wrote_planes = pk == R29 and not pout32
        assert (src == PLANES) == wrote_planes, (k, rounds)
        if kernel == R29:
            assert bool(in32) == (src == WORDS)
        else:
            assert src == WORDS


def test_plan_of_the_shape_that_once_faulted():
    """D = 2^12, N = 2^4 from two integer columns: round 0 is the first-round kernel
    reading the integers, round 1 the 29-bit kernel folding them, every later round
    reads the workspace."""
    import paper_2404_16109_amd as zk
    rc, rounds = _plan(zk, 1 << 12, 1 << 4, from_ints=True)
    assert rc == 12
    assert rounds[0][:2] == (FIRST, INTS)
    assert rounds[1][:3] == (R29, INTS, 1)
    # pairs 1024 (round 1) and 512 (round 2) run on 29-bit limbs, 256 to 64 pairs in the resident kernel, the rest on the host
    assert [r[0] for r in rounds] == [FIRST, R29, R29] + [RESIDENT] * 3 + [HOST] * 6
    assert rounds[2][1] == PLANES and rounds[2][3] == 1      # reads planes, writes words for the resident kernel
    assert all(r[1] == WORDS for r in rounds[3:])
    _check_chain(rounds)
    # the same shape from a vector: the first pass serves two rounds, the third binds both variables from the caller's S
    rc, from_vec = _plan(zk, 1 << 12, 1 << 4)
    assert [r[0] for r in from_vec] == [FIRST_TWO, NO_PASS, R29] + [RESIDENT] * 3 + [HOST] * 6
    assert [r[1] for r in from_vec[:3]] == [CALLER] * 3 and from_vec[2][2:] == (1, 1) and from_vec[3:] == rounds[3:]
    _check_chain(from_vec)


def test_plan_of_the_headline_shape_matches_the_bench_model():
    import bench
    import paper_2404_16109_amd as zk
    for from_ints in (False, True):
        rc, rounds = _plan(zk, 1 << 25, 1 << 16, from_ints=from_ints)
        assert rc == 25
        assert [k for k, r in enumerate(rounds) if r[0] == R29] == bench.rounds_on_29_bits(1 << 25, 1 << 16, from_ints)
        assert [r[0] for r in rounds[9:16]] == [BOTH] * 7 and [r[0] for r in rounds[16:]] == [RESIDENT] * 3 + [HOST] * 6
        # eight folds at most before reduced words are written again: the first 29-bit round arrives as words, round 8
        # leaves as words
        first29 = 1 if from_ints else 2
        assert rounds[first29][2] == 1 and rounds[8][3] == 1 and all(r[3] == 0 for r in rounds[first29:8])
        assert (rounds[0][0], rounds[1][0]) == ((FIRST, R29) if from_ints else (FIRST_TWO, NO_PASS))
        _check_chain(rounds)


def test_every_shape_has_a_kernel_for_every_round():
    import paper_2404_16109_amd as zk
    for n in range(0, 23):
        for l in range(0, n + 1):
            D, N = 1 << n, 1 << l
            for K in (1, 2):
                rc, rounds = _plan(zk, D, N, K)
                assert rc == n
                _check_chain(rounds)
                if K == 2:
                    assert all(r[0] not in (RESIDENT, HOST) for r in rounds)
                # the host's rounds: the last ones, at most 32 pairs each, and only after the resident kernel has run
                kinds = [r[0] for r in rounds]
                if HOST in kinds:
                    first = kinds.index(HOST)
                    assert first >= 1 and kinds[first - 1] == RESIDENT and kinds[first:] == [HOST] * (n - first)
                    assert first == max(n - 6, kinds.index(RESIDENT) + 1)
                elif RESIDENT in kinds:
                    assert kinds.index(RESIDENT) == n - 1  # the resident kernel's only round is the last one
            rc, rounds = _plan(zk, D, N, from_ints=True)
            takes_ints = zk.tlookup_small_workspace_bytes(D, N) == -(-zk.tlookup_workspace_bytes(D, N) // 256) * 256
            if rc < 0:
                # no integer path for this shape: tlookup_prove_small writes S out first and needs room for it
                assert rc == zk.ZK_E_BADARG and not takes_ints
                continue
            assert takes_ints and N <= 1 << 16 and D >= 4 * N and D > 1024
            assert rounds[0][:2] == (FIRST, INTS) and rounds[1][:3] == (R29, INTS, 1)
            assert all(r[1] in (WORDS, PLANES) for r in rounds[2:])
            _check_chain(rounds)


def test_plan_argument_errors():
    import paper_2404_16109_amd as zk
    assert _plan(zk, 1000, 8)[0] == zk.ZK_E_BADARG
    assert _plan(zk, 8, 16)[0] == zk.ZK_E_BADARG
    assert _plan(zk, 1 << 12, 1 << 4, K=2, from_ints=True)[0] == zk.ZK_E_BADARG
    assert _plan(zk, 1 << 12, 1 << 4, K=9)[0] == zk.ZK_E_BADARG
