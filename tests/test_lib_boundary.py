"""CPU-side checks of the device library's boundary: it loads, exports every
function the header declares, its host-only verifier agrees with the oracle, and
argument errors are reported without touching a GPU."""
import re

import numpy as np


def _declared_functions():
    text = open("include/zkmi.h").read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"^(?:int|size_t)\s+(\w+)\s*\(", text, flags=re.M)))


def test_library_exports_every_declared_function():
    import paper_2404_16109_amd as zk
    names = _declared_functions()
    assert len(names) >= 30
    for name in names:
        assert hasattr(zk.raw(), name), name
        assert name in zk.EXPORTS, name
    assert zk.zkmi_version() >= 100


def test_constants_match_python():
    import paper_2404_16109_amd as zk
    from tests.pyref import R
    rc, mod, r1, r2, ninv = zk.fr_constants()
    assert (rc, mod, r1, r2, ninv) == (0, R, 2 ** 256 % R, 2 ** 512 % R, (-pow(R, -1, 2 ** 32)) % 2 ** 32)


def test_sizes():
    import paper_2404_16109_amd as zk
    assert zk.tlookup_proof_bytes(1 << 25) == 280 + 128 * 25
    assert zk.tlookup_proof_bytes(1) == 280
    assert zk.tlookup_workspace_bytes(1 << 10, 1 << 8) > 0
    assert zk.tlookup_workspace_bytes(1000, 256) == 0
    assert zk.raw().sumcheck_product_proof_bytes(8) == 16 + 32 + 3 * 96 + 64
    assert zk.raw().matmul_proof_bytes(5120) == 64 + 13 * 96 + 64


def test_host_verifier_accepts_oracle_product_proofs(orc):
    """The library's host-only product-sumcheck verifier replays proofs written by
    the oracle: transcript, interpolation and field code of the two sides agree."""
    import random
    import paper_2404_16109_amd as zk
    from tests.pyref import R
    rng = random.Random(77)
    for d in (0, 1, 4, 7):
        a = [rng.randrange(R) for _ in range(1 << d)]
        b = [rng.randrange(R) for _ in range(1 << d)]
        claim = sum(x * y for x, y in zip(a, b)) % R
        seed = rng.randbytes(32)
        rc, proof, r = orc.sumcheck_prove_product(seed, orc.to_bytes(a), orc.to_bytes(b), orc.to_bytes([claim])[0])
        assert rc == 0
        rc, fin, pt = zk.sumcheck_verify_product(seed, proof, 1 << d)
        assert rc == zk.ZK_OK
        assert pt == orc.to_ints(r)
        assert fin == [int.from_bytes(proof[-64:-32], "little"), int.from_bytes(proof[-32:], "little")]
        if d:
            for pos in rng.sample(range(len(proof)), 30):
                bad = bytearray(proof)
                bad[pos] ^= 1 << rng.randrange(8)
                assert zk.sumcheck_verify_product(seed, bytes(bad), 1 << d)[0] == zk.ZK_E_REJECT
        assert zk.sumcheck_verify_product(seed, proof, 3)[0] == zk.ZK_E_BADARG


def test_library_sha256_both_paths_match_hashlib():
    """The transcript's hash, through the portable compression function and through
    the x86 SHA extensions (when the processor has them), against hashlib at every
    length around the block and padding boundaries, and on long inputs."""
    import hashlib
    import random
    import paper_2404_16109_amd as zk
    rng = random.Random(9)
    lengths = list(range(0, 200)) + [255, 256, 257, 1000, 4096, 16384, 16385]
    used_any = False
    for n in lengths:
        data = rng.randbytes(n)
        want = hashlib.sha256(data).digest()
        used, got = zk.zkmi_sha256(data, use_sha_instructions=False)
        assert used == 0 and got == want, n
        used, got = zk.zkmi_sha256(data, use_sha_instructions=True)
        assert used in (0, 1) and got == want, n
        used_any = used_any or used == 1
    golden = [l.split() for l in open("tests/golden/sha256_vectors.txt") if l.strip() and not l.startswith("#")]
    assert golden
    for message, digest in golden:
        for flag in (False, True):
            assert zk.zkmi_sha256(message.encode(), use_sha_instructions=flag)[1].hex() == digest
    cpu_has_sha = "sha_ni" in open("/proc/cpuinfo").read()
    assert used_any == cpu_has_sha


def test_host_verifier_accepts_oracle_link_proofs(orc):
    """The library's verifier of the zkAttn linking sumcheck, without tensors (no
    GPU involved), replays proofs written by the oracle and rejects corrupted ones."""
    import random
    import paper_2404_16109_amd as zk
    from tests.test_oracle_link import make_witness, prove
    rng = random.Random(78)
    for rows, cols, K in [(1, 1, 1), (2, 4, 2), (8, 4, 3), (4, 16, 2)]:
        w = make_witness(rng, rows, cols, K)
        seed = rng.randbytes(32)
        rc, proof, point = prove(orc, seed, w, rows, cols)
        assert rc == 0
        rc, claims = zk.zkattn_link_verify(seed, proof, rows, cols, w[5])
        assert rc == zk.ZK_OK and claims["v"] == orc.to_ints(point)
        n = (rows * cols).bit_length() - 1
        fin = [int.from_bytes(proof[64 + n * (K + 2) * 32 + 32 * q:][:32], "little") for q in range(2 * K + 2)]
        assert [claims["Zp_v"]] + claims["X_v"] + [claims["Y_v"]] + claims["Yk_v"] == fin
        for pos in rng.sample(range(len(proof)), min(40, len(proof))):
            bad = bytearray(proof)
            bad[pos] ^= 1 << rng.randrange(8)
            assert zk.zkattn_link_verify(seed, bytes(bad), rows, cols, w[5])[0] == zk.ZK_E_REJECT
        assert zk.zkattn_link_verify(seed, proof, rows, cols, [b + 1 for b in w[5]])[0] == zk.ZK_E_REJECT
