"""Pins of the oracle's SHA-256 and transcript framing (no GPU)."""
import hashlib
import random

from tests import pyref


def test_sha256_published_vectors(orc):
    for line in open("tests/golden/sha256_vectors.txt"):
        if not line.strip() or line.startswith("#"):
            continue
        msg, digest = line.split()
        assert orc.sha256(msg.encode()).hex() == digest


def test_sha256_against_hashlib(orc):
    rng = random.Random(1)
    for n in list(range(0, 200)) + [255, 256, 257, 1000, 4096, 65537]:
        data = rng.randbytes(n)
        assert orc.sha256(data) == hashlib.sha256(data).digest(), n


def test_transcript_framing(orc):
    rng = random.Random(2)
    init = b"zkmi/test" + rng.randbytes(32)
    a, b = orc.Transcript(init), pyref.Transcript(init)
    assert a.state.tobytes() == b.state
    for step in range(20):
        if step % 3 == 0:
            data = rng.randbytes(rng.randrange(0, 300))
            a.absorb("g", data)
            b.absorb("g", data)
        else:
            tag = rng.choice(["beta", "alpha", "u", "r"])
            assert orc.to_ints(a.challenge(tag)) == [b.challenge(tag)]
        assert a.state.tobytes() == b.state


def test_pair_combiner(orc):
    seed = bytes(range(32))
    t = pyref.Transcript(b"zkmi/rho/v1" + seed)
    assert orc.to_ints(orc.pair_combiner(seed)) == [t.challenge("rho")]
