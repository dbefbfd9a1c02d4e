"""Brute-force definitions in Python big integers, for tiny cases only.

This is the yardstick the CPU oracle is pinned against: every function is the
definition in the paper evaluated term by term (Section 3.3 for multilinear
extensions and sumcheck rounds, Section 4 for the tlookup summand), with
`hashlib` as the hash.  Cost is exponential; keep n <= 5.
"""
import hashlib
import itertools

Z = -0xd201000000010000
R = Z ** 4 - Z ** 2 + 1          # BLS12-381 scalar field order


def bits_msb_first(x, n):
    return [(x >> (n - 1 - t)) & 1 for t in range(n)]


def eq(u, w):
    """e~(u, w) = prod_t (u_t w_t + (1-u_t)(1-w_t)) for field points u, w."""
    acc = 1
    for a, b in zip(u, w):
        acc = acc * ((a * b + (1 - a) * (1 - b)) % R) % R
    return acc


def mle(arr, point):
    """arr~(point) = sum_x e~(point, bits(x)) arr[x]; point[0] is the top index bit."""
    n = len(point)
    assert len(arr) == 1 << n
    return sum(eq(point, bits_msb_first(x, n)) * arr[x] for x in range(1 << n)) % R


class Transcript:
    def __init__(self, init):
        self.state = hashlib.sha256(init).digest()

    def absorb(self, tag, data):
        self.state = hashlib.sha256(self.state + tag.encode() + len(data).to_bytes(8, "little") + data).digest()

    def challenge(self, tag):
        t = tag.encode()
        h0 = hashlib.sha256(self.state + t + b"\x00").digest()
        h1 = hashlib.sha256(self.state + t + b"\x01").digest()
        self.state = hashlib.sha256(self.state + t + b"\x02").digest()
        return int.from_bytes(h0 + h1, "big") % R


def fr_bytes(x):
    return int(x % R).to_bytes(32, "little")


def m_digest(counts, leaf=128):
    leaves = b""
    for base in range(0, len(counts), leaf):
        leaves += hashlib.sha256(b"".join(int(c).to_bytes(4, "little") for c in counts[base:base + leaf])).digest()
    return hashlib.sha256(leaves).digest()


def vec_digest(vals, leaf=128):
    """Hash tree over a vector of field elements: leaf i holds elements i, i+L, i+2L, ...
    (L = n/leaf leaves, one leaf when n < leaf); rows of digests are then hashed in
    consecutive fours (a last pair in twos) down to one digest."""
    n = len(vals)
    L = max(1, n // leaf)
    row = [hashlib.sha256(b"".join(fr_bytes(vals[x]) for x in range(i, n, L))).digest() for i in range(L)]
    while len(row) > 1:
        g = 4 if len(row) >= 4 else 2
        row = [hashlib.sha256(b"".join(row[i:i + g])).digest() for i in range(0, len(row), g)]
    return row[0]


def round_poly(f, prefix, nvars, X):
    """g_k(X) = sum over rest in {0,1}^(nvars-k-1) of f(prefix, X, rest)."""
    k = len(prefix)
    total = 0
    for rest in itertools.product((0, 1), repeat=nvars - k - 1):
        total += f(list(prefix) + [X] + list(rest))
    return total % R


def tlookup_proof(seed, S, T):
    """The whole tlookup proof from the definitions; S, T lists of ints mod R."""
    D, N = len(S), len(T)
    n, l = D.bit_length() - 1, N.bit_length() - 1
    h = n - l
    first = {}
    for j, t in enumerate(T):
        first.setdefault(t, j)
    m = [0] * N
    for s in S:
        m[first[s]] += 1
    tr = Transcript(b"zkmi/tlookup/v2" + seed + D.to_bytes(8, "little") + N.to_bytes(8, "little"))
    md = m_digest(m)
    tr.absorb("m", md)
    beta = tr.challenge("beta")
    A = [pow(beta + s, -1, R) for s in S]
    B = [pow(beta + t, -1, R) for t in T]
    dA, dB = vec_digest(A), vec_digest(B)
    tr.absorb("A", dA)
    tr.absorb("B", dB)
    alpha = tr.challenge("alpha")
    u = [tr.challenge("u") for _ in range(n)]
    scale = pow(pow(2, h, R), -1, R)

    def f(w):
        wt = w[h:]
        left = mle(A, w) * ((alpha * eq(u, w) % R) * ((mle(S, w) + beta) % R) + 1) % R
        right = scale * mle(B, wt) % R * ((alpha * alpha % R) * eq(u[h:], wt) % R * ((mle(T, wt) + beta) % R) - mle(m, wt)) % R
        return (left + right) % R

    out = b"ZKTL" + (2).to_bytes(4, "little") + D.to_bytes(8, "little") + N.to_bytes(8, "little") + md + dA + dB
    v = []
    polys = []
    for k in range(n):
        g = [round_poly(f, v, n, X) for X in range(5)]
        polys.append(g)
        msg = b"".join(fr_bytes(y) for y in g[:4])
        out += msg
        tr.absorb("g", msg)
        v.append(tr.challenge("r"))
    vt = v[h:]
    fin = [mle(A, v), mle(S, v), mle(B, vt), mle(m, vt), mle(T, vt)]
    out += b"".join(fr_bytes(y) for y in fin)
    return out, {"beta": beta, "alpha": alpha, "u": u, "v": v, "m": m, "A": A, "B": B, "polys": polys, "f": f}


def _ceil_log2(v):
    return max((v - 1).bit_length(), 0)


def product_rounds(tr, a, b):
    """Rounds of sum_x a(x) b(x) from the definition; returns (bytes, challenges)."""
    d = len(a).bit_length() - 1
    f = lambda w: mle(a, w) * mle(b, w) % R
    out, r = b"", []
    for k in range(d):
        g = [round_poly(f, r, d, X) for X in range(3)]
        msg = b"".join(fr_bytes(y) for y in g)
        out += msg
        tr.absorb("g", msg)
        r.append(tr.challenge("r"))
    fin = fr_bytes(mle(a, r)) + fr_bytes(mle(b, r))
    tr.absorb("final", fin)
    return out + fin, r


def product_proof(seed, a, b, claim):
    d = len(a).bit_length() - 1
    tr = Transcript(b"zkmi/sumcheck-product/v1" + seed + d.to_bytes(8, "little"))
    tr.absorb("claim", fr_bytes(claim))
    body, r = product_rounds(tr, a, b)
    return b"ZKSP" + (1).to_bytes(4, "little") + d.to_bytes(8, "little") + fr_bytes(claim) + body, r


def matmul_proof(seed, X, W):
    """X, W: lists of rows of Python ints (signed).  Everything from the definitions:
    the claim is the multilinear extension of the integer product X W at (u, v)."""
    D0, D1, D2 = len(X), len(W), len(W[0])
    n0, n1, n2 = _ceil_log2(D0), _ceil_log2(D1), _ceil_log2(D2)
    tr = Transcript(b"zkmi/matmul/v1" + seed + b"".join(d.to_bytes(8, "little") for d in (D0, D1, D2)))
    u = [tr.challenge("u") for _ in range(n0)]
    v = [tr.challenge("v") for _ in range(n2)]
    Y = [[sum(X[i][k] * W[k][j] for k in range(D1)) for j in range(D2)] for i in range(D0)]

    def padded(M, rows, cols, nr, nc):
        flat = [0] * ((1 << nr) * (1 << nc))
        for i in range(rows):
            for j in range(cols):
                flat[i * (1 << nc) + j] = M[i][j] % R
        return flat

    claim = mle(padded(Y, D0, D2, n0, n2), u + v)
    Xp, Wp = padded(X, D0, D1, n0, n1), padded(W, D1, D2, n1, n2)
    a = [mle(Xp, u + bits_msb_first(k, n1)) for k in range(1 << n1)]
    b = [mle(Wp, bits_msb_first(k, n1) + v) for k in range(1 << n1)]
    tr.absorb("claim", fr_bytes(claim))
    body, r = product_rounds(tr, a, b)
    head = b"ZKMM" + (1).to_bytes(4, "little") + b"".join(d.to_bytes(8, "little") for d in (D0, D1, D2))
    return head + fr_bytes(claim) + body, {"u": u, "v": v, "r": r, "claim": claim, "Y": Y,
                                           "Xr": mle(Xp, u + r), "Wr": mle(Wp, r + v)}


def tlookup_batch_proof(seed, S_list, T_list):
    """K tlookup instances of one shape under one sumcheck of f = sum_k lambda^k f_k,
    everything from the definitions."""
    K, D, N = len(S_list), len(S_list[0]), len(T_list[0])
    n, l = D.bit_length() - 1, N.bit_length() - 1
    h = n - l
    tr = Transcript(b"zkmi/tlookup-batch/v2" + seed + D.to_bytes(8, "little") + N.to_bytes(8, "little") + K.to_bytes(8, "little"))
    out = b"ZKTB" + (2).to_bytes(4, "little") + D.to_bytes(8, "little") + N.to_bytes(8, "little") + K.to_bytes(8, "little")
    ms = []
    for S, T in zip(S_list, T_list):
        first = {}
        for j, t in enumerate(T):
            first.setdefault(t, j)
        m = [0] * N
        for s in S:
            m[first[s]] += 1
        ms.append(m)
        md = m_digest(m)
        tr.absorb("m", md)
        out += md
    beta = tr.challenge("beta")
    As = [[pow(beta + s, -1, R) for s in S] for S in S_list]
    Bs = [[pow(beta + t, -1, R) for t in T] for T in T_list]
    for A, B in zip(As, Bs):
        dA, dB = vec_digest(A), vec_digest(B)
        tr.absorb("A", dA)
        tr.absorb("B", dB)
        out += dA + dB
    alpha = tr.challenge("alpha")
    u = [tr.challenge("u") for _ in range(n)]
    lam = tr.challenge("lambda")
    scale = pow(pow(2, h, R), -1, R)

    def f(w):
        wt = w[h:]
        total = 0
        for k in range(K):
            A, S, B, T, m = As[k], S_list[k], Bs[k], T_list[k], ms[k]
            left = mle(A, w) * ((alpha * eq(u, w) % R) * ((mle(S, w) + beta) % R) + 1) % R
            right = scale * mle(B, wt) % R * ((alpha * alpha % R) * eq(u[h:], wt) % R * ((mle(T, wt) + beta) % R) - mle(m, wt)) % R
            total += pow(lam, k, R) * (left + right)
        return total % R

    v = []
    first_claim = None
    for k in range(n):
        g = [round_poly(f, v, n, X) for X in range(4)]
        if first_claim is None:
            first_claim = (g[0] + g[1]) % R
        msg = b"".join(fr_bytes(y) for y in g)
        out += msg
        tr.absorb("g", msg)
        v.append(tr.challenge("r"))
    vt = v[h:]
    fin = b""
    for k in range(K):
        fin += b"".join(fr_bytes(y) for y in [mle(As[k], v), mle(S_list[k], v), mle(Bs[k], vt), mle(ms[k], vt), mle(T_list[k], vt)])
    out += fin
    return out, {"beta": beta, "alpha": alpha, "lambda": lam, "v": v, "first_claim": first_claim, "m": ms}


def tlookup_multi_proof(seed, S_list, T_list):
    """K tlookup instances of any shapes (D_k, N_k) under one sumcheck over n = max_k log2 D_k
    variables.  Instance k lives on the last n_k = log2 D_k of them and its summand does not
    depend on the first n - n_k: f = sum_k lambda^k 2^-(n - n_k) f_k(w[n - n_k:]), f_k built on
    u[n - n_k:].  Everything from the definitions."""
    K = len(S_list)
    Ds, Ns = [len(S) for S in S_list], [len(T) for T in T_list]
    ns = [D.bit_length() - 1 for D in Ds]
    hs = [ns[k] - (Ns[k].bit_length() - 1) for k in range(K)]
    n = max(ns)
    init = b"zkmi/tlookup-multi/v1" + seed + K.to_bytes(8, "little")
    out = b"ZKTM" + (1).to_bytes(4, "little") + K.to_bytes(8, "little")
    for D, N in zip(Ds, Ns):
        init += D.to_bytes(8, "little") + N.to_bytes(8, "little")
        out += D.to_bytes(8, "little") + N.to_bytes(8, "little")
    tr = Transcript(init)
    ms = []
    for S, T in zip(S_list, T_list):
        first = {}
        for j, t in enumerate(T):
            first.setdefault(t, j)
        m = [0] * len(T)
        for s in S:
            m[first[s]] += 1
        ms.append(m)
        md = m_digest(m)
        tr.absorb("m", md)
        out += md
    beta = tr.challenge("beta")
    As = [[pow(beta + s, -1, R) for s in S] for S in S_list]
    Bs = [[pow(beta + t, -1, R) for t in T] for T in T_list]
    for A, B in zip(As, Bs):
        dA, dB = vec_digest(A), vec_digest(B)
        tr.absorb("A", dA)
        tr.absorb("B", dB)
        out += dA + dB
    alpha = tr.challenge("alpha")
    u = [tr.challenge("u") for _ in range(n)]
    lam = tr.challenge("lambda")

    def f(w):
        total = 0
        for k in range(K):
            skip = n - ns[k]
            wk, uk = w[skip:], u[skip:]
            wt, ut = wk[hs[k]:], uk[hs[k]:]
            A, S, B, T, m = As[k], S_list[k], Bs[k], T_list[k], ms[k]
            left = mle(A, wk) * ((alpha * eq(uk, wk) % R) * ((mle(S, wk) + beta) % R) + 1) % R
            right = pow(pow(2, hs[k], R), -1, R) * mle(B, wt) % R * ((alpha * alpha % R) * eq(ut, wt) % R * ((mle(T, wt) + beta) % R) - mle(m, wt)) % R
            total += pow(lam, k, R) * pow(pow(2, skip, R), -1, R) % R * (left + right)
        return total % R

    v, polys = [], []
    for k in range(n):
        g = [round_poly(f, v, n, X) for X in range(4)]
        polys.append(g)
        msg = b"".join(fr_bytes(y) for y in g)
        out += msg
        tr.absorb("g", msg)
        v.append(tr.challenge("r"))
    fin = b""
    for k in range(K):
        vk = v[n - ns[k]:]
        vt = vk[hs[k]:]
        fin += b"".join(fr_bytes(y) for y in [mle(As[k], vk), mle(S_list[k], vk), mle(Bs[k], vt), mle(ms[k], vt), mle(T_list[k], vt)])
    out += fin
    return out, {"beta": beta, "alpha": alpha, "lambda": lam, "v": v, "polys": polys, "m": ms}


def zkattn_link_proof(seed, Zp, X, Y, Yk, yhat, bases, rows, cols):
    """The sumcheck linking zkAttn's tensors (Protocol 2, last step) from the
    definitions: every round polynomial is the sum of the summand, built from
    brute-force multilinear extensions, over the remaining cube.  Lists of ints."""
    K = len(X)
    nr, nc = rows.bit_length() - 1, cols.bit_length() - 1
    n = nr + nc
    init = b"zkmi/zkattn-link/v1" + seed + rows.to_bytes(8, "little") + cols.to_bytes(8, "little") + K.to_bytes(8, "little")
    init += b"".join(fr_bytes(b) for b in bases)
    tr = Transcript(init)
    u = [tr.challenge("u") for _ in range(n)]
    cy = mle(yhat, u[:nr])
    tr.absorb("yhat", fr_bytes(cy))
    alpha = tr.challenge("alpha")

    def f(w):
        lin = mle(Zp, w)
        prod = 1
        for k in range(K):
            lin += bases[k] * mle(X[k], w)
            prod = prod * mle(Yk[k], w) % R
        y = mle(Y, w)
        return (eq(u, w) * ((lin + alpha * (y - prod)) % R) + alpha * alpha % R * eq(u[:nr], w[:nr]) % R * y) % R

    out = b"ZKAL" + (1).to_bytes(4, "little") + rows.to_bytes(8, "little") + cols.to_bytes(8, "little") + K.to_bytes(8, "little")
    out += fr_bytes(cy)
    v, polys = [], []
    for k in range(n):
        g = [round_poly(f, v, n, Xp) for Xp in range(K + 4)]
        polys.append(g)
        msg = b"".join(fr_bytes(y) for y in g[:K + 2])
        out += msg
        tr.absorb("g", msg)
        v.append(tr.challenge("r"))
    fin = [mle(Zp, v)] + [mle(X[k], v) for k in range(K)] + [mle(Y, v)] + [mle(Yk[k], v) for k in range(K)]
    out += b"".join(fr_bytes(y) for y in fin)
    return out, {"u": u, "alpha": alpha, "cy": cy, "v": v, "polys": polys, "f": f, "fin": fin}
