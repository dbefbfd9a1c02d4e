"""Seeded synthetic inputs shared by the device path, the tests and the bench.

Nothing here does any of the method's arithmetic: the functions return plain
integer arrays (values, table columns, table-row indices); embedding them in
the field, combining pair tables and everything after that is done separately
by each implementation.

The workloads imitate, in shape and value range, the tensors of the paper's
experiments (Section 8: sequence length 2048, fixed-point scale 2^16, tables of
2^16 rows), whose real activations and weights are not available here.

Random stream: SplitMix64 used as a counter-based generator, value i of stream
`seed` is mix(seed + (i+1)*0x9E3779B97F4A7C15).
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)


def splitmix64(seed, n, offset=0):
    """n 64-bit values of stream `seed`, starting at counter `offset`."""
    with np.errstate(over="ignore"):
        i = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
        z = np.uint64(seed) + i * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def uniform_ints(seed, n, lo, hi):
    """n integers uniform in [lo, hi) as int64."""
    span = np.uint64(hi - lo)
    return (splitmix64(seed, n) % span).astype(np.int64) + np.int64(lo)


def _unit_open(bits):
    # (0, 1): 53 random bits, shifted off zero
    return ((bits >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def rounded_normal(seed, n, sigma, lo, hi, chunk=1 << 24):
    """round-half-away-from-zero of N(0, sigma^2) samples (Box-Muller), clipped to [lo, hi)."""
    out = np.empty(n, dtype=np.int64)
    for start in range(0, n, chunk):
        m = min(chunk, n - start)
        u1 = _unit_open(splitmix64(seed, m, offset=2 * start))
        u2 = _unit_open(splitmix64(seed, m, offset=2 * start + m))
        g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2) * float(sigma)
        r = np.sign(g) * np.floor(np.abs(g) + 0.5)
        out[start:start + m] = np.clip(r, lo, hi - 1).astype(np.int64)
    return out


def seed_bytes(tag):
    """32-byte transcript seed for a named workload."""
    raw = splitmix64(int.from_bytes(tag.encode()[:8].ljust(8, b"\0"), "little"), 4)
    return raw.astype("<u8").tobytes()


def range_check_unsigned(D=1 << 10, N=1 << 8, seed=1):
    """Config 1: S uniform in [0, N), table (0 .. N-1)."""
    idx = uniform_ints(seed, D, 0, N).astype(np.uint32)
    tx = np.arange(N, dtype=np.int64)
    return {"name": "c1-range-u8", "D": D, "N": N, "idx": idx, "tx": tx, "ty": None,
            "seed": seed_bytes("c1")}


def range_check_signed(D=1 << 20, N=1 << 8, seed=2):
    """Config 2: S uniform in [-N/2, N/2), table (-N/2 .. N/2-1); negative values embed as r-|x|."""
    x = uniform_ints(seed, D, -(N // 2), N // 2)
    tx = np.arange(-(N // 2), N // 2, dtype=np.int64)
    return {"name": "c2-range-i8", "D": D, "N": N, "idx": (x + N // 2).astype(np.uint32), "tx": tx, "ty": None,
            "seed": seed_bytes("c2")}


def activation_table(rows=2048, cols=11008, logD=25, logN=16, sigma=None, seed=3):
    """Config 3: activations ~ rounded N(0, sigma) clipped to the table's input
    range, looked up in an input/output pair table; the tensor is padded to 2^logD
    entries with copies of table row 0."""
    N, D = 1 << logN, 1 << logD
    half = N // 2
    sigma = (N / 16.0) if sigma is None else sigma          # 2^12 at N = 2^16
    real = min(rows * cols, D)
    x = rounded_normal(seed, real, sigma, -half, half)
    idx = np.zeros(D, dtype=np.uint32)
    idx[:real] = (x + half).astype(np.uint32)
    tx = np.arange(-half, half, dtype=np.int64)
    ty = uniform_ints(seed + 1000, N, -half, half)
    return {"name": "c3-activation", "D": D, "N": N, "idx": idx, "tx": tx, "ty": ty, "real": real,
            "seed": seed_bytes("c3")}


def matmul_operands(D0=2048, D1=5120, D2=5120, sigma_x=256.0, sigma_w=64.0, seed=4):
    """Config 4: int16 fixed-point operands of Y = X W."""
    X = rounded_normal(seed, D0 * D1, sigma_x, -(1 << 15), 1 << 15).reshape(D0, D1)
    W = rounded_normal(seed + 1000, D1 * D2, sigma_w, -(1 << 15), 1 << 15).reshape(D1, D2)
    return {"name": "c4-matmul", "X": X, "W": W, "seed": seed_bytes("c4")}


def attention_segments(heads=40, rows=2048, cols=2048, logD=28, logN=16, sigma=65536.0, seed=5):
    """Config 5: attention scores minus their row maximum (<= 0), negated and
    split into two base-2^logN digits; each digit is looked up in its own pair
    table.  Returns one instance per digit."""
    N, D = 1 << logN, 1 << logD
    real = heads * rows * cols
    assert real <= D
    z = rounded_normal(seed, real, sigma, -(1 << 31), 1 << 31).reshape(heads * rows, cols)
    z = (z.max(axis=1, keepdims=True) - z).reshape(-1)           # -(z - rowmax) >= 0
    z = np.minimum(z, N * N - 1)
    out = []
    for k in range(2):
        digit = ((z >> (logN * k)) & (N - 1)).astype(np.uint32)
        idx = np.zeros(D, dtype=np.uint32)
        idx[:real] = digit
        tx = np.arange(N, dtype=np.int64)
        ty = uniform_ints(seed + 1000 * (k + 1), N, 0, 1 << 16)
        out.append({"name": "c5-attn-seg%d" % k, "D": D, "N": N, "idx": idx, "tx": tx, "ty": ty, "real": real,
                    "seed": seed_bytes("c5s%d" % k)})
    return out


def attention_link(heads=40, rows=2048, cols=2048, logN=16, sigma=65536.0, seed=5):
    """Config 5, the tensors that zkAttn's closing sumcheck links: the same scores
    and digit tables as attention_segments, as a (heads*rows padded to a power of
    two) x cols matrix.  Returns the digits x[k] and the table columns ty[k] (the
    segment outputs are ty[k][x[k]], their product and its row sums follow from
    them); padded rows hold the digit 0."""
    N = 1 << logN
    real_rows = heads * rows
    prows = 1
    while prows < real_rows:
        prows <<= 1
    z = rounded_normal(seed, real_rows * cols, sigma, -(1 << 31), 1 << 31).reshape(real_rows, cols)
    z = (z.max(axis=1, keepdims=True) - z).reshape(-1)
    z = np.minimum(z, N * N - 1)
    x, ty = [], []
    for k in range(2):
        digit = np.zeros(prows * cols, dtype=np.uint32)
        digit[:real_rows * cols] = ((z >> (logN * k)) & (N - 1)).astype(np.uint32)
        x.append(digit)
        ty.append(uniform_ints(seed + 1000 * (k + 1), N, 0, 1 << 16))
    return {"name": "c5-attn-link", "rows": prows, "cols": cols, "x": x, "ty": ty, "bases": [1, N],
            "seed": seed_bytes("c5link")}


BLS12_381_R = 0x73eda753299d7d483339d80809a1d80553bda402fffe5bfeffffffff00000001


def pair_combiner(seed):
    """The verifier's random combiner rho of a pair table (an input to both
    implementations): a hash of the workload seed, reduced into the field."""
    import hashlib
    st = hashlib.sha256(b"zkmi/rho/v1" + bytes(seed)).digest()
    wide = hashlib.sha256(st + b"rho\x00").digest() + hashlib.sha256(st + b"rho\x01").digest()
    return int.from_bytes(wide, "big") % BLS12_381_R
