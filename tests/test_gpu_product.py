"""GPU parity: product sumcheck and the matmul proof (Section 6.1.1) through the C
boundary against the CPU oracle, byte for byte."""
import random

import numpy as np
import pytest
import torch

from paper_2404_16109_amd import synth
from tests.pyref import R

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def zk():
    import paper_2404_16109_amd as zk
    assert torch.cuda.is_available()
    return zk


@pytest.mark.parametrize("d", [0, 1, 2, 5, 11, 13, 16])
def test_product_sumcheck(zk, orc, d):
    rng = random.Random(200 + d)
    n = 1 << d
    mask = np.array([255] * 31 + [63], dtype=np.uint8)
    A = np.frombuffer(rng.randbytes(32 * n), dtype=np.uint8).reshape(n, 32) & mask
    B = np.frombuffer(rng.randbytes(32 * n), dtype=np.uint8).reshape(n, 32) & mask
    claim = orc.to_ints(orc.fr_sum(orc.fr_mul(A, B)))[0]
    seed = rng.randbytes(32)
    rc_o, want, r = orc.sumcheck_prove_product(seed, A, B, orc.to_bytes([claim])[0])
    va, vb = zk.vec_from_bytes(A), zk.vec_from_bytes(B)
    rc, got = zk.sumcheck_prove_product(seed, va, vb, claim)
    assert rc == 0 == rc_o and got == want
    rc, fin, pt = zk.sumcheck_verify_product(seed, got, n)
    assert rc == 0 and pt == orc.to_ints(r)
    # the final values are the multilinear extensions at the point
    assert fin[0] == orc.to_ints(orc.mle_eval(A, r))[0] if d else fin[0] == orc.to_ints(A)[0]


def _matmul_case(zk, orc, X, W, seed):
    D0, D1 = X.shape
    D2 = W.shape[1]
    rc_o, want, info = orc.matmul_sumcheck_prove(seed, X, W)
    vx, vw = zk.Vec(D0 * D1), zk.Vec(D1 * D2)
    assert zk.fr_from_i32(vx, torch.from_numpy(X.astype(np.int32).reshape(-1)).cuda()) == 0
    assert zk.fr_from_i32(vw, torch.from_numpy(W.astype(np.int32).reshape(-1)).cuda()) == 0
    rc, got = zk.matmul_sumcheck_prove(seed, vx, D0, D1, vw, D2)
    assert rc == 0 == rc_o
    assert got == want
    # the same bytes straight from the 16-bit matrices
    if np.abs(X).max() < 1 << 15 and np.abs(W).max() < 1 << 15:
        rc, got16 = zk.matmul_sumcheck_prove_i16(seed, torch.from_numpy(X.astype(np.int16)).cuda(),
                                                 torch.from_numpy(W.astype(np.int16)).cuda())
        assert rc == 0 and got16 == want
    return got, vx, vw


@pytest.mark.parametrize("shape", [(1, 1, 1), (2, 3, 2), (4, 4, 4), (3, 5, 6), (8, 7, 2), (37, 300, 65), (128, 1024, 96)])
def test_matmul_proof(zk, orc, shape):
    D0, D1, D2 = shape
    rng = np.random.default_rng(300 + D0 + D1 + D2)
    X = rng.integers(-300, 300, (D0, D1))
    W = rng.integers(-100, 100, (D1, D2))
    seed = bytes(rng.integers(0, 256, 32, dtype=np.uint8))
    proof, vx, vw = _matmul_case(zk, orc, X, W, seed)
    Y = X.astype(np.int64) @ W.astype(np.int64)
    vy = zk.Vec(D0 * D2)
    assert zk.fr_from_i32(vy, torch.from_numpy(Y.astype(np.int32).reshape(-1)).cuda()) == 0
    assert zk.matmul_sumcheck_verify(seed, proof, D0, D1, D2) == 0
    assert zk.matmul_sumcheck_verify(seed, proof, D0, D1, D2, Y=vy, X=vx, W=vw) == 0
    assert orc.matmul_sumcheck_verify(seed, proof, D0, D1, D2, Y=orc.fr_from_i64(Y.reshape(-1)), X=X, W=W) == 0
    Y2 = Y.copy()
    Y2[-1, -1] += 1
    vy2 = zk.Vec(D0 * D2)
    assert zk.fr_from_i32(vy2, torch.from_numpy(Y2.astype(np.int32).reshape(-1)).cuda()) == 0
    assert zk.matmul_sumcheck_verify(seed, proof, D0, D1, D2, Y=vy2) == zk.ZK_E_REJECT
    if len(proof) > 200:
        bad = bytearray(proof)
        bad[150] ^= 2
        assert zk.matmul_sumcheck_verify(seed, bytes(bad), D0, D1, D2) == zk.ZK_E_REJECT


def test_config4_matmul_13b_layer_shape(zk, orc):
    cfg = synth.matmul_operands()
    _matmul_case(zk, orc, cfg["X"], cfg["W"], cfg["seed"])


def test_matmul_i16_extreme_values(zk, orc):
    """Entries at both ends of the 16-bit range, all of one sign, and columns of
    zeros: the unreduced accumulators take their largest values."""
    rng = np.random.default_rng(77)
    D0, D1, D2 = 300, 40, 129
    for fill in (-32768, 32767):
        X = np.full((D0, D1), fill, dtype=np.int64)
        W = np.full((D1, D2), fill, dtype=np.int64)
        X[:, 3] = 0
        W[5, :] = -fill - 1 if fill < 0 else -fill
        seed = bytes(rng.integers(0, 256, 32, dtype=np.uint8))
        rc_o, want, _ = orc.matmul_sumcheck_prove(seed, X, W)
        rc, got = zk.matmul_sumcheck_prove_i16(seed, torch.from_numpy(X.astype(np.int16)).cuda(),
                                               torch.from_numpy(W.astype(np.int16)).cuda())
        assert rc == 0 == rc_o and got == want


def test_resident_kernel_gives_up_when_the_host_is_silent(zk, orc):
    """The bounded wait of the kernels that receive challenges from the host, forced
    from the host side: a tiny bound, no answer; the kernel ends by itself.  A proof
    made right after it is unaffected."""
    assert zk.zkmi_selftest_resident_wait() == zk.ZK_OK
    rng = random.Random(99)
    a = [rng.randrange(R) for _ in range(64)]
    b = [rng.randrange(R) for _ in range(64)]
    claim = sum(x * y for x, y in zip(a, b)) % R
    va, vb = zk.vec_from_bytes(orc.to_bytes(a)), zk.vec_from_bytes(orc.to_bytes(b))
    rc, proof = zk.sumcheck_prove_product(b"\x03" * 32, va, vb, claim)
    assert rc == 0 and zk.sumcheck_verify_product(b"\x03" * 32, proof, 64)[0] == 0
