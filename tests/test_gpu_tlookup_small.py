"""tlookup_prove_small on the GPU: the tensor given as signed 32-bit integers, alone
(a range check) or as two columns combined by rho (Section 4's reduction of a
function table to a set), must give tlookup_prove's proof of S = X + rho Y byte
for byte, which in turn is the oracle's; shapes on either side of the path that
never writes S out; extreme integers; duplicates in the table; a wrong entry is
found and reported by its index."""
import random

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
R = 0x73eda753299d7d483339d80809a1d80553bda402fffe5bfeffffffff00000001


@pytest.fixture(scope="module")
def zk():
    import paper_2404_16109_amd as zk
    assert torch.cuda.is_available()
    return zk


def i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def make(gen, D, N, paired, lo=-(1 << 31), hi=1 << 31, dup=False):
    """A table of N rows of small integers (pairs if `paired`), D looked-up rows, rho."""
    tx = gen.integers(lo, hi, N)
    ty = gen.integers(lo, hi, N) if paired else None
    if dup and N >= 4:
        tx[N - 1] = tx[1]
        tx[2] = tx[1]
        if paired:
            ty[N - 1] = ty[1]
            ty[2] = ty[1]
    rho = int(gen.integers(1, 1 << 62)) * int(gen.integers(1, 1 << 62)) * int(gen.integers(1, 1 << 62)) % R if paired else None
    idx = gen.integers(0, N, D)
    return tx, ty, rho, idx


def field(values, rho_values=None, rho=0):
    out = [int(v) % R for v in values]
    if rho_values is not None:
        out = [(a + rho * int(b)) % R for a, b in zip(out, rho_values)]
    return out


@pytest.mark.parametrize("D,N,paired", [
    (1 << 12, 1 << 4, True), (1 << 12, 1 << 10, False),      # the first fold is a kernel of its own: S is never written out
    (1 << 15, 1 << 8, True), (1 << 16, 1 << 14, False), (1 << 17, 1 << 15, True), (1 << 18, 1, False),
    (1 << 10, 1 << 4, True), (1 << 12, 1 << 11, False), (64, 8, True), (1 << 13, 1 << 13, False), (2, 1, True)])  # written out first
def test_same_proof_as_from_field_elements(zk, orc, D, N, paired):
    gen = np.random.default_rng(D * 7 + N + paired)
    tx, ty, rho, idx = make(gen, D, N, paired, dup=(D + N) % 3 == 0)
    Tb = orc.to_bytes(field(tx, ty, rho or 0))
    Sb = Tb[idx]
    seed = bytes(gen.integers(0, 256, 32, dtype=np.uint8))
    rc_o, want, _ = orc.tlookup_prove(seed, Sb, Tb)
    assert rc_o == 0
    Tv = zk.vec_from_bytes(Tb)
    X, Y = i32(tx[idx]), i32(ty[idx]) if paired else None
    rc, got, info = zk.tlookup_prove_small(seed, X, Y, rho, i32(idx), Tv)
    assert rc == zk.ZK_OK and got == want and info["sum_A"] == info["sum_mB"]
    rc, again, _ = zk.tlookup_prove(seed, zk.vec_from_bytes(Sb), i32(idx), Tv)
    assert rc == zk.ZK_OK and again == got


def test_extreme_integers(zk, orc):
    """Entries at both ends of the 32-bit range and zero, with rho = r - 1 and rho = 1."""
    D, N = 1 << 12, 8
    gen = np.random.default_rng(5)
    edge = np.array([-(1 << 31), (1 << 31) - 1, 0, -1, 1, -(1 << 31) + 1, 12345, -54321])
    for rho in (R - 1, 1, 2):
        tx, ty = edge, edge[::-1].copy()
        idx = gen.integers(0, N, D)
        Tb = orc.to_bytes(field(tx, ty, rho))
        Sb = Tb[idx]
        seed = bytes(gen.integers(0, 256, 32, dtype=np.uint8))
        rc_o, want, _ = orc.tlookup_prove(seed, Sb, Tb)
        rc, got, _ = zk.tlookup_prove_small(seed, i32(tx[idx]), i32(ty[idx]), rho, i32(idx), zk.vec_from_bytes(Tb))
        assert rc_o == 0 and rc == zk.ZK_OK and got == want


def test_a_wrong_entry_is_reported(zk, orc):
    gen = np.random.default_rng(6)
    for D, N in ((1 << 13, 1 << 6), (1 << 9, 1 << 4)):   # with and without the path that never writes S out
        tx, ty, rho, idx = make(gen, D, N, True, lo=-1000, hi=1000)
        Tv = zk.vec_from_bytes(orc.to_bytes(field(tx, ty, rho)))
        x, y = tx[idx].copy(), ty[idx].copy()
        for pos, which in ((D - 3, "x"), (5, "y"), (D // 2, "x")):
            bx, by = x.copy(), y.copy()
            (bx if which == "x" else by)[pos] += 1
            rc, proof, info = zk.tlookup_prove_small(b"\x05" * 32, i32(bx), i32(by), rho, i32(idx), Tv)
            assert rc == zk.ZK_E_NOT_IN_TABLE and proof == b"" and info["bad_index"] == pos


def test_argument_errors(zk, orc):
    gen = np.random.default_rng(8)
    D, N = 1 << 12, 1 << 4
    tx, ty, rho, idx = make(gen, D, N, True)
    Tv = zk.vec_from_bytes(orc.to_bytes(field(tx, ty, rho)))
    X, Y, I = i32(tx[idx]), i32(ty[idx]), i32(idx)
    seed = b"\x01" * 32
    assert zk.tlookup_prove_small(seed, X, Y, rho, None, Tv)[0] == zk.ZK_E_BADARG       # hints are required
    assert zk.tlookup_prove_small(seed, X, Y, None, I, Tv)[0] == zk.ZK_E_BADARG         # a second column without rho
    assert zk.tlookup_prove_small(seed, X, None, rho, I, Tv)[0] == zk.ZK_E_BADARG       # rho without a second column
    assert zk.tlookup_prove_small(seed, X, Y, R, I, Tv)[0] == zk.ZK_E_BADARG            # rho not canonical
    assert zk.tlookup_prove_small(seed, X[:3000], Y[:3000], rho, I, Tv)[0] == zk.ZK_E_BADARG   # not a power of two
    assert zk.tlookup_prove_small(seed, X, Y, rho, I, Tv, cap=16)[0] == zk.ZK_E_BUFSZ
    small_ws = torch.empty(1024, dtype=torch.uint8, device="cuda")
    assert zk.tlookup_prove_small(seed, X, Y, rho, I, Tv, ws=small_ws)[0] == zk.ZK_E_BUFSZ
