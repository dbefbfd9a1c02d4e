"""The seeded input generators (paper_2404_16109_amd/synth.py), on the CPU: the
random stream is SplitMix64 as published (checked against a scalar
re-implementation on Python integers and its well-known first output for seed
zero), the draws are reproducible, and each workload has the shape, ranges and
structure its recipe states: uniform range checks, a clipped rounded-normal
activation tensor padded with row 0, int16 matmul operands, and attention scores
split into two digits of which the high one takes only a handful of values."""
import numpy as np

from paper_2404_16109_amd import synth

MASK = (1 << 64) - 1


def splitmix64_scalar(seed, n):
    """SplitMix64 (Steele, Lea, Flood 2014; Vigna's reference code): the state advances
    by the golden-ratio constant, the output is the state mixed twice."""
    out, state = [], seed & MASK
    for _ in range(n):
        state = (state + 0x9E3779B97F4A7C15) & MASK
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
        out.append(z ^ (z >> 31))
    return out


def test_random_stream_is_splitmix64():
    assert int(synth.splitmix64(0, 1)[0]) == 0xE220A8397B1DCDAF        # first output of the reference code for seed 0
    for seed in (0, 1, 5, 0xDEADBEEFCAFEF00D, MASK):
        assert [int(v) for v in synth.splitmix64(seed, 50)] == splitmix64_scalar(seed, 50)
    # a stream can be entered anywhere
    whole = synth.splitmix64(7, 1000)
    assert np.array_equal(synth.splitmix64(7, 300, offset=700), whole[700:])


def test_draws_are_reproducible_and_in_range():
    a = synth.uniform_ints(3, 10000, -5, 17)
    assert np.array_equal(a, synth.uniform_ints(3, 10000, -5, 17)) and a.min() == -5 and a.max() == 16
    assert not np.array_equal(a, synth.uniform_ints(4, 10000, -5, 17))
    g = synth.rounded_normal(9, 200000, 100.0, -250, 250)
    assert np.array_equal(g, synth.rounded_normal(9, 200000, 100.0, -250, 250))
    assert g.min() == -250 and g.max() == 249                        # clipped to [lo, hi)
    inner = g[(g > -250) & (g < 249)]
    assert abs(inner.mean()) < 1.0 and 90.0 < g.std() < 100.0        # sigma 100, tails cut at 2.5 sigma
    assert len(synth.seed_bytes("c3")) == 32 and synth.seed_bytes("c3") != synth.seed_bytes("c4")
    rho = synth.pair_combiner(synth.seed_bytes("c3"))
    assert 0 < rho < synth.BLS12_381_R and rho == synth.pair_combiner(synth.seed_bytes("c3"))


def test_range_check_workloads():
    c1 = synth.range_check_unsigned()
    assert (c1["D"], c1["N"]) == (1 << 10, 1 << 8) and c1["idx"].dtype == np.uint32 and len(c1["idx"]) == c1["D"]
    assert c1["idx"].max() < c1["N"] and np.array_equal(c1["tx"], np.arange(256)) and c1["ty"] is None
    c2 = synth.range_check_signed(D=1 << 12)
    assert np.array_equal(c2["tx"], np.arange(-128, 128)) and c2["idx"].max() < 256
    assert len(np.unique(c2["idx"])) == 256                          # every row is hit: 256 hot bins


def test_activation_workload_structure():
    c3 = synth.activation_table(rows=8, cols=100, logD=10, logN=8)
    D, N = 1 << 10, 1 << 8
    assert (c3["D"], c3["N"], c3["real"]) == (D, N, 800) and len(c3["idx"]) == D
    assert np.all(c3["idx"][800:] == 0)                               # padded with table row 0
    assert c3["idx"].max() < N
    x = c3["idx"][:800].astype(np.int64) - N // 2                     # the activations themselves
    assert abs(x.mean()) < 3.0 and 12.0 < x.std() < 20.0              # sigma = N / 16 = 16
    assert np.array_equal(c3["tx"], np.arange(-N // 2, N // 2)) and len(c3["ty"]) == N
    assert c3["ty"].min() >= -N // 2 and c3["ty"].max() < N // 2
    # the tensor is longer than the real activations only by padding; a full one is cut at D
    full = synth.activation_table(rows=64, cols=64, logD=10, logN=8)
    assert full["real"] == D


def test_matmul_operands():
    c4 = synth.matmul_operands(D0=16, D1=64, D2=32)
    assert c4["X"].shape == (16, 64) and c4["W"].shape == (64, 32)
    for m in (c4["X"], c4["W"]):
        assert m.min() >= -(1 << 15) and m.max() < (1 << 15)
    assert 150.0 < c4["X"].std() < 350.0 and 40.0 < c4["W"].std() < 90.0


def test_attention_workloads():
    segs = synth.attention_segments(heads=2, rows=16, cols=64, logD=12, logN=8, sigma=300.0)
    assert len(segs) == 2 and all(s["D"] == 1 << 12 and s["N"] == 1 << 8 for s in segs)
    real = 2 * 16 * 64
    lo, hi = segs[0]["idx"][:real].astype(np.int64), segs[1]["idx"][:real].astype(np.int64)
    z = lo + (hi << 8)                                                # row maximum minus score
    assert z.min() == 0 and np.all(z.reshape(32, 64).min(axis=1) == 0)   # every row attains its maximum
    assert len(np.unique(hi)) <= 12 and len(np.unique(lo)) > 100      # a dozen hot bins in the high digit
    assert np.all(segs[0]["idx"][real:] == 0) and segs[0]["seed"] != segs[1]["seed"]
    link = synth.attention_link(heads=3, rows=16, cols=64, logN=8, sigma=300.0)
    assert (link["rows"], link["cols"]) == (64, 64) and link["bases"] == [1, 256]   # 48 rows padded to 64
    assert all(len(x) == 64 * 64 and x.max() < 256 for x in link["x"]) and np.all(link["x"][0][48 * 64:] == 0)
    assert all(len(t) == 256 and t.min() >= 0 and t.max() < (1 << 16) for t in link["ty"])
