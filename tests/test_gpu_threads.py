"""Two host threads proving at the same time, each on a stream and a workspace of its own: the library's host state
(the pinned memory kernels report into, the channel a resident kernel reads its challenges from) is per thread, so
the proofs must come out as they do alone.  bench.py times this arrangement beside the headline."""
import random
import threading

import numpy as np
import pytest
import torch

from tests.pyref import R

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def zk():
    import paper_2404_16109_amd as zk
    assert torch.cuda.is_available()
    return zk


def _instance(orc, zk, rng, D, N):
    T, seen = [], set()
    while len(T) < N:
        t = rng.randrange(R)
        if t not in seen:
            seen.add(t)
            T.append(t)
    rows = np.random.default_rng(rng.randrange(1 << 30)).integers(0, N, size=D)
    tb = orc.to_bytes(T)
    sb = tb[rows]
    return sb, tb, zk.vec_from_bytes(sb), zk.vec_from_bytes(tb), torch.from_numpy(rows.astype(np.int32)).cuda()


def test_two_threads_prove_at_once(zk, orc):
    rng = random.Random(4242)
    # two different lookups: one with rounds on 29-bit limbs and the resident kernel, one small
    cases = [_instance(orc, zk, rng, 1 << 17, 1 << 6), _instance(orc, zk, rng, 1 << 14, 1 << 9)]
    seeds = [rng.randbytes(32), rng.randbytes(32)]
    want = []
    for (sb, tb, _, _, _), seed in zip(cases, seeds):
        rc, proof, _ = orc.tlookup_prove(seed, sb, tb)
        assert rc == 0
        want.append(proof)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    got = [[], []]
    errors = []

    def worker(which):
        try:
            _, _, S, T, idx = cases[which]
            with torch.cuda.stream(streams[which]):
                for _ in range(6):
                    rc, proof, _ = zk.tlookup_prove(seeds[which], S, idx, T)
                    got[which].append((rc, proof))
        except Exception as e:  # surfaced below: a thread must not fail silently
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(w,)) for w in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for which in range(2):
        assert len(got[which]) == 6
        for rc, proof in got[which]:
            assert rc == 0 and proof == want[which]


def test_thread_state_can_be_made_and_given_back(zk, orc):
    """zkmi_thread_init allocates the calling thread's pinned state ahead of the first proof; zkmi_thread_release frees
    it, after which the next call allocates it again: proofs are the same before, between and after."""
    rng = random.Random(99)
    sb, tb, S, T, idx = _instance(orc, zk, rng, 1 << 13, 1 << 9)
    seed = rng.randbytes(32)
    rc, want, _ = orc.tlookup_prove(seed, sb, tb)
    assert rc == 0

    def worker(out):
        try:
            out.append(zk.zkmi_thread_init(1 << 9))
            out.append(zk.tlookup_prove(seed, S, idx, T)[:2])
            out.append(zk.zkmi_thread_release())
            out.append(zk.zkmi_thread_release())             # nothing left to free: still fine
            out.append(zk.tlookup_prove(seed, S, idx, T)[:2])  # allocates again by itself
            out.append(zk.zkmi_thread_release())
        except Exception as e:
            out.append(repr(e))

    got = []
    t = threading.Thread(target=worker, args=(got,))
    t.start()
    t.join()
    torch.cuda.synchronize()
    assert got == [0, (0, want), 0, 0, (0, want), 0]
    # the main thread's own state is untouched by another thread's release
    assert zk.tlookup_prove(seed, S, idx, T)[:2] == (0, want)
