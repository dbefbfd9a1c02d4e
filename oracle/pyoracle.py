"""CPU oracle -- TEST INFRASTRUCTURE, not the product.

ctypes binding of ``liboracle.so`` (built from ``capi.cpp`` by :func:`build`).
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module; the device library never does.

Field elements are numpy ``uint8`` arrays of shape ``(..., 32)``: the 32
little-endian bytes of the canonical integer in ``[0, r)``.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

OK, E_BADARG, E_NOT_IN_TABLE, E_ZERO_DENOM, E_REJECT, E_BUFSZ = 0, -1, -2, -3, -4, -5


def build(force=True):
    """Compile the oracle with the host compiler."""
    if not force and os.path.exists(_LIB_PATH):
        return _LIB_PATH
    cmd = ["g++", "-O2", "-std=c++17", "-Wall", "-shared", "-fPIC", "-pthread",
           os.path.join(_HERE, "capi.cpp"), "-o", _LIB_PATH]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.oracle_tlookup_proof_bytes.restype = ctypes.c_uint64
        _lib.oracle_product_proof_bytes.restype = ctypes.c_uint64
        _lib.oracle_tlookup_batch_proof_bytes.restype = ctypes.c_uint64
        _lib.oracle_tlookup_multi_proof_bytes.restype = ctypes.c_uint64
        _lib.oracle_matmul_proof_bytes.restype = ctypes.c_uint64
        _lib.oracle_link_proof_bytes.restype = ctypes.c_uint64
    return _lib


def default_threads():
    return max(1, min(16, os.cpu_count() or 1))


# ---- conversions -----------------------------------------------------------

def to_bytes(values):
    """Python ints in [0, r) -> uint8 array (len, 32)."""
    out = np.zeros((len(values), 32), dtype=np.uint8)
    for i, v in enumerate(values):
        out[i] = np.frombuffer(int(v).to_bytes(32, "little"), dtype=np.uint8)
    return out


def to_ints(arr):
    arr = np.ascontiguousarray(arr, dtype=np.uint8).reshape(-1, 32)
    return [int.from_bytes(row.tobytes(), "little") for row in arr]


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _c(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.uint8)


def _u64(x):
    return ctypes.c_uint64(int(x))


# ---- field -----------------------------------------------------------------

def modulus():
    out = np.zeros(32, dtype=np.uint8)
    lib().oracle_fr_modulus(_p(out))
    return int.from_bytes(out.tobytes(), "little")


def barrett_mu():
    out = np.zeros(40, dtype=np.uint8)
    lib().oracle_fr_barrett_mu(_p(out))
    return int.from_bytes(out.tobytes(), "little")


def _binary(name, a, b):
    a, b = _c(a).reshape(-1, 32), _c(b).reshape(-1, 32)
    assert a.shape == b.shape
    out = np.empty_like(a)
    getattr(lib(), name)(_p(out), _p(a), _p(b), _u64(a.shape[0]))
    return out


def fr_add(a, b):
    return _binary("oracle_fr_add", a, b)


def fr_sub(a, b):
    return _binary("oracle_fr_sub", a, b)


def fr_mul(a, b):
    return _binary("oracle_fr_mul", a, b)


def fr_axpy(x, s, y=None, threads=None):
    """x + s*y elementwise (y None: x + s)."""
    x = _c(x).reshape(-1, 32)
    y = None if y is None else _c(y).reshape(-1, 32)
    out = np.empty_like(x)
    lib().oracle_fr_axpy(_p(out), _p(x), _p(_c(s)), _p(y), _u64(x.shape[0]), threads or default_threads())
    return out


def fr_mul_scalar(x, s):
    x = _c(x).reshape(-1, 32)
    out = np.empty_like(x)
    lib().oracle_fr_mul_scalar(_p(out), _p(x), _p(_c(s)), _u64(x.shape[0]))
    return out


def fr_inv(a, threads=None):
    a = _c(a).reshape(-1, 32)
    out = np.zeros_like(a)
    rc = lib().oracle_fr_inv(_p(out), _p(a), _u64(a.shape[0]), threads or default_threads())
    return rc, out


def fr_pow(a, e):
    out = np.zeros(32, dtype=np.uint8)
    ee = np.frombuffer(int(e).to_bytes(32, "little"), dtype=np.uint8).copy()
    lib().oracle_fr_pow(_p(out), _p(_c(a)), _p(ee))
    return out


def fr_sum(a):
    a = _c(a).reshape(-1, 32)
    out = np.zeros(32, dtype=np.uint8)
    lib().oracle_fr_sum(_p(out), _p(a), _u64(a.shape[0]))
    return out


def fr_from_i64(x):
    x = np.ascontiguousarray(x, dtype=np.int64).reshape(-1)
    out = np.empty((x.shape[0], 32), dtype=np.uint8)
    lib().oracle_fr_from_i64(_p(out), x.ctypes.data_as(ctypes.c_void_p), _u64(x.shape[0]))
    return out


def fr_from_be512(b64):
    buf = np.frombuffer(bytes(b64), dtype=np.uint8).copy()
    assert buf.shape[0] == 64
    out = np.zeros(32, dtype=np.uint8)
    lib().oracle_fr_from_be512(_p(out), _p(buf))
    return out


def all_canonical(a):
    a = _c(a).reshape(-1, 32)
    return bool(lib().oracle_fr_all_canonical(_p(a), _u64(a.shape[0])))


# ---- hash / transcript -----------------------------------------------------

def sha256(data):
    buf = np.frombuffer(bytes(data), dtype=np.uint8).copy() if len(data) else np.zeros(1, dtype=np.uint8)
    out = np.zeros(32, dtype=np.uint8)
    lib().oracle_sha256(_p(out), _p(buf), _u64(len(data)))
    return out.tobytes()


class Transcript:
    def __init__(self, init_bytes):
        self.state = np.zeros(32, dtype=np.uint8)
        buf = np.frombuffer(bytes(init_bytes), dtype=np.uint8).copy()
        lib().oracle_transcript_init(_p(self.state), _p(buf), _u64(len(init_bytes)))

    def absorb(self, tag, data):
        buf = np.frombuffer(bytes(data), dtype=np.uint8).copy() if len(data) else np.zeros(1, dtype=np.uint8)
        lib().oracle_transcript_absorb(_p(self.state), tag.encode(), _p(buf), _u64(len(data)))

    def challenge(self, tag):
        out = np.zeros(32, dtype=np.uint8)
        lib().oracle_transcript_challenge(_p(self.state), tag.encode(), _p(out))
        return out


def pair_combiner(seed):
    out = np.zeros(32, dtype=np.uint8)
    lib().oracle_pair_combiner(_p(_c(np.frombuffer(bytes(seed), dtype=np.uint8))), _p(out))
    return out


# ---- polynomials -----------------------------------------------------------

def eq_table(u, threads=None):
    u = _c(u).reshape(-1, 32)
    n = u.shape[0]
    out = np.empty((1 << n, 32), dtype=np.uint8)
    lib().oracle_eq_table(_p(out), _p(u), n, threads or default_threads())
    return out


def eq_at_point(u, v):
    u, v = _c(u).reshape(-1, 32), _c(v).reshape(-1, 32)
    out = np.zeros(32, dtype=np.uint8)
    lib().oracle_eq_at_point(_p(out), _p(u), _p(v), u.shape[0])
    return out


def mle_eval(s, point, threads=None):
    s, point = _c(s).reshape(-1, 32), _c(point).reshape(-1, 32)
    assert s.shape[0] == 1 << point.shape[0]
    out = np.zeros(32, dtype=np.uint8)
    lib().oracle_mle_eval(_p(out), _p(s), point.shape[0], _p(point), threads or default_threads())
    return out


def lagrange_eval(y, at):
    y = _c(y).reshape(-1, 32)
    out = np.zeros(32, dtype=np.uint8)
    lib().oracle_lagrange_eval(_p(out), _p(y), y.shape[0], _p(_c(at)))
    return out


# ---- tlookup ---------------------------------------------------------------

def multiplicities(S, T, threads=None):
    S, T = _c(S).reshape(-1, 32), _c(T).reshape(-1, 32)
    m = np.zeros(T.shape[0], dtype=np.uint64)
    bad = ctypes.c_uint64(0)
    rc = lib().oracle_multiplicities(m.ctypes.data_as(ctypes.c_void_p), _p(S), _u64(S.shape[0]), _p(T),
                                     _u64(T.shape[0]), ctypes.byref(bad), threads or default_threads())
    return rc, m, bad.value


def m_digest(m):
    m = np.ascontiguousarray(m, dtype=np.uint64)
    out = np.zeros(32, dtype=np.uint8)
    lib().oracle_m_digest(_p(out), m.ctypes.data_as(ctypes.c_void_p), _u64(m.shape[0]))
    return out.tobytes()


def vec_digest(v, threads=None):
    """Digest of a vector of field elements (canonical bytes, n a power of two)."""
    v = _c(v).reshape(-1, 32)
    out = np.zeros(32, dtype=np.uint8)
    lib().oracle_vec_digest(_p(out), _p(v), _u64(v.shape[0]), threads or default_threads())
    return out.tobytes()


def tlookup_proof_bytes(D):
    return int(lib().oracle_tlookup_proof_bytes(_u64(D)))


def tlookup_prove(seed, S, T, forced_beta=None, threads=None, cap=None):
    """Returns (rc, proof bytes, info dict)."""
    S, T = _c(S).reshape(-1, 32), _c(T).reshape(-1, 32)
    D, N = S.shape[0], T.shape[0]
    n = max(D.bit_length() - 1, 0)
    size = tlookup_proof_bytes(D) if D and (D & (D - 1)) == 0 else 64
    cap = size if cap is None else cap
    proof = np.zeros(max(cap, 1), dtype=np.uint8)
    ln = ctypes.c_uint64(0)
    aux = np.zeros((4, 32), dtype=np.uint8)
    u = np.zeros((max(n, 1), 32), dtype=np.uint8)
    v = np.zeros((max(n, 1), 32), dtype=np.uint8)
    bad = ctypes.c_uint64(0)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    fb = None if forced_beta is None else _c(forced_beta)
    rc = lib().oracle_tlookup_prove(_p(seedb), _p(S), _u64(D), _p(T), _u64(N), _p(proof), _u64(cap),
                                    ctypes.byref(ln), _p(aux), _p(u), _p(v), ctypes.byref(bad), _p(fb),
                                    threads or default_threads())
    info = {"len": ln.value, "beta": aux[0], "alpha": aux[1], "sum_A": aux[2], "sum_mB": aux[3],
            "u": u[:n], "v": v[:n], "bad_index": bad.value}
    return rc, proof[:ln.value].tobytes() if rc == OK else b"", info


def tlookup_verify(seed, proof, T, D, S=None, m=None, A=None, B=None, threads=None):
    """Returns (rc, info dict with claims, point v and failing stage)."""
    T = _c(T).reshape(-1, 32)
    N = T.shape[0]
    n = max(int(D).bit_length() - 1, 0)
    pb = np.frombuffer(bytes(proof), dtype=np.uint8).copy() if len(proof) else np.zeros(1, dtype=np.uint8)
    claims = np.zeros((5, 32), dtype=np.uint8)
    v = np.zeros((max(n, 1), 32), dtype=np.uint8)
    stage = ctypes.c_int(0)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    mm = None if m is None else np.ascontiguousarray(m, dtype=np.uint64)
    rc = lib().oracle_tlookup_verify(_p(seedb), _p(pb), _u64(len(proof)), _p(T), _u64(D), _u64(N),
                                     _p(None if S is None else _c(S).reshape(-1, 32)),
                                     None if mm is None else mm.ctypes.data_as(ctypes.c_void_p),
                                     _p(None if A is None else _c(A).reshape(-1, 32)),
                                     _p(None if B is None else _c(B).reshape(-1, 32)),
                                     _p(claims), _p(v), ctypes.byref(stage), threads or default_threads())
    return rc, {"claims": claims, "v": v[:n], "stage": stage.value}


def _ptr_array(arrays):
    arr = (ctypes.c_void_p * len(arrays))()
    for i, a in enumerate(arrays):
        arr[i] = None if a is None else a.ctypes.data
    return arr


def tlookup_batch_prove(seed, S_list, T_list, threads=None):
    """Several instances of one shape, one sumcheck.  Returns (rc, proof, info)."""
    S_list = [_c(s).reshape(-1, 32) for s in S_list]
    T_list = [_c(t).reshape(-1, 32) for t in T_list]
    K, D, N = len(S_list), S_list[0].shape[0], T_list[0].shape[0]
    n = max(D.bit_length() - 1, 0)
    cap = int(lib().oracle_tlookup_batch_proof_bytes(_u64(D), _u64(K))) if D and (D & (D - 1)) == 0 else 64
    proof = np.zeros(cap, dtype=np.uint8)
    ln = ctypes.c_uint64(0)
    aux = np.zeros((3 + 2 * K, 32), dtype=np.uint8)
    v = np.zeros((max(n, 1), 32), dtype=np.uint8)
    bad_i, bad_x = ctypes.c_uint64(0), ctypes.c_uint64(0)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    rc = lib().oracle_tlookup_batch_prove(_p(seedb), _ptr_array(S_list), _ptr_array(T_list), _u64(K), _u64(D), _u64(N),
                                          _p(proof), _u64(cap), ctypes.byref(ln), _p(aux), _p(v), ctypes.byref(bad_i),
                                          ctypes.byref(bad_x), threads or default_threads())
    info = {"beta": aux[0], "alpha": aux[1], "lambda": aux[2], "sum_A": aux[3::2], "sum_mB": aux[4::2], "v": v[:n],
            "bad_instance": bad_i.value, "bad_index": bad_x.value}
    return rc, proof[:ln.value].tobytes() if rc == OK else b"", info


def tlookup_batch_verify(seed, proof, T_list, D, S_list=None, m_list=None, threads=None):
    T_list = [_c(t).reshape(-1, 32) for t in T_list]
    K, N = len(T_list), T_list[0].shape[0]
    pb = np.frombuffer(bytes(proof), dtype=np.uint8).copy() if len(proof) else np.zeros(1, dtype=np.uint8)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    S_arr = None if S_list is None else _ptr_array([_c(s).reshape(-1, 32) for s in S_list])
    keep_m = None if m_list is None else [np.ascontiguousarray(m, dtype=np.uint64) for m in m_list]
    m_arr = None if keep_m is None else _ptr_array(keep_m)
    keep_s = None if S_list is None else [_c(s).reshape(-1, 32) for s in S_list]
    S_arr = None if keep_s is None else _ptr_array(keep_s)
    return lib().oracle_tlookup_batch_verify(_p(seedb), _p(pb), _u64(len(proof)), _ptr_array(T_list), _u64(K), _u64(D),
                                             _u64(N), S_arr, m_arr, None, threads or default_threads())


def tlookup_multi_prove(seed, S_list, T_list, threads=None):
    """Several instances of any shapes, one sumcheck.  Returns (rc, proof, info)."""
    S_list = [_c(s).reshape(-1, 32) for s in S_list]
    T_list = [_c(t).reshape(-1, 32) for t in T_list]
    K = len(S_list)
    Ds = np.array([s.shape[0] for s in S_list], dtype=np.uint64)
    Ns = np.array([t.shape[0] for t in T_list], dtype=np.uint64)
    n = max(max(int(d).bit_length() - 1, 0) for d in Ds)
    cap = int(lib().oracle_tlookup_multi_proof_bytes(_u64(n), _u64(K)))
    proof = np.zeros(cap, dtype=np.uint8)
    ln = ctypes.c_uint64(0)
    aux = np.zeros((3 + 2 * K, 32), dtype=np.uint8)
    v = np.zeros((max(n, 1), 32), dtype=np.uint8)
    bad_i, bad_x = ctypes.c_uint64(0), ctypes.c_uint64(0)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    rc = lib().oracle_tlookup_multi_prove(_p(seedb), _ptr_array(S_list), _ptr_array(T_list), _u64(K), _p(Ds), _p(Ns),
                                          _p(proof), _u64(cap), ctypes.byref(ln), _p(aux), _p(v), ctypes.byref(bad_i),
                                          ctypes.byref(bad_x), threads or default_threads())
    info = {"beta": aux[0], "alpha": aux[1], "lambda": aux[2], "sum_A": aux[3::2], "sum_mB": aux[4::2], "v": v[:n],
            "bad_instance": bad_i.value, "bad_index": bad_x.value}
    return rc, proof[:ln.value].tobytes() if rc == OK else b"", info


def tlookup_multi_verify(seed, proof, T_list, D_list, S_list=None, m_list=None, threads=None):
    T_list = [_c(t).reshape(-1, 32) for t in T_list]
    K = len(T_list)
    Ds = np.array([int(d) for d in D_list], dtype=np.uint64)
    Ns = np.array([t.shape[0] for t in T_list], dtype=np.uint64)
    pb = np.frombuffer(bytes(proof), dtype=np.uint8).copy() if len(proof) else np.zeros(1, dtype=np.uint8)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    keep_m = None if m_list is None else [None if m is None else np.ascontiguousarray(m, dtype=np.uint64) for m in m_list]
    m_arr = None if keep_m is None else _ptr_array(keep_m)
    keep_s = None if S_list is None else [None if s is None else _c(s).reshape(-1, 32) for s in S_list]
    S_arr = None if keep_s is None else _ptr_array(keep_s)
    return lib().oracle_tlookup_multi_verify(_p(seedb), _p(pb), _u64(len(proof)), _ptr_array(T_list), _u64(K), _p(Ds),
                                             _p(Ns), S_arr, m_arr, None, threads or default_threads())


# ---- product sumcheck / matmul ----------------------------------------------

def sumcheck_prove_product(seed, a, b, claim, threads=None):
    a, b = _c(a).reshape(-1, 32), _c(b).reshape(-1, 32)
    n = a.shape[0]
    d = n.bit_length() - 1
    cap = int(lib().oracle_product_proof_bytes(_u64(n)))
    proof = np.zeros(cap, dtype=np.uint8)
    ln = ctypes.c_uint64(0)
    r = np.zeros((max(d, 1), 32), dtype=np.uint8)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    rc = lib().oracle_sumcheck_prove_product(_p(seedb), _p(a), _p(b), _u64(n), _p(_c(claim)), _p(proof),
                                             _u64(cap), ctypes.byref(ln), _p(r), threads or default_threads())
    return rc, proof[:ln.value].tobytes() if rc == OK else b"", r[:d]


def sumcheck_verify_product(seed, proof, n, a=None, b=None, threads=None):
    pb = np.frombuffer(bytes(proof), dtype=np.uint8).copy() if len(proof) else np.zeros(1, dtype=np.uint8)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    return lib().oracle_sumcheck_verify_product(_p(seedb), _p(pb), _u64(len(proof)), _u64(n),
                                                _p(None if a is None else _c(a).reshape(-1, 32)),
                                                _p(None if b is None else _c(b).reshape(-1, 32)), None,
                                                threads or default_threads())


def matmul_sumcheck_prove(seed, X, W, threads=None):
    """X: (D0, D1) int64, W: (D1, D2) int64.  Returns (rc, proof, info)."""
    X = np.ascontiguousarray(X, dtype=np.int64)
    W = np.ascontiguousarray(W, dtype=np.int64)
    D0, D1 = X.shape
    D2 = W.shape[1]
    assert W.shape[0] == D1
    cap = int(lib().oracle_matmul_proof_bytes(_u64(D1)))
    proof = np.zeros(cap, dtype=np.uint8)
    ln = ctypes.c_uint64(0)
    n0, n1, n2 = [max((int(d) - 1).bit_length(), 0) for d in (D0, D1, D2)]
    u = np.zeros((max(n0, 1), 32), dtype=np.uint8)
    v = np.zeros((max(n2, 1), 32), dtype=np.uint8)
    r = np.zeros((max(n1, 1), 32), dtype=np.uint8)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    rc = lib().oracle_matmul_sumcheck_prove(_p(seedb), X.ctypes.data_as(ctypes.c_void_p), _u64(D0), _u64(D1),
                                            W.ctypes.data_as(ctypes.c_void_p), _u64(D2), _p(proof), _u64(cap),
                                            ctypes.byref(ln), _p(u), _p(v), _p(r), threads or default_threads())
    return rc, proof[:ln.value].tobytes() if rc == OK else b"", {"u": u[:n0], "v": v[:n2], "r": r[:n1]}


def matmul_sumcheck_verify(seed, proof, D0, D1, D2, Y=None, X=None, W=None, threads=None):
    pb = np.frombuffer(bytes(proof), dtype=np.uint8).copy() if len(proof) else np.zeros(1, dtype=np.uint8)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    Xc = None if X is None else np.ascontiguousarray(X, dtype=np.int64)
    Wc = None if W is None else np.ascontiguousarray(W, dtype=np.int64)
    return lib().oracle_matmul_sumcheck_verify(
        _p(seedb), _p(pb), _u64(len(proof)), _u64(D0), _u64(D1), _u64(D2),
        _p(None if Y is None else _c(Y).reshape(-1, 32)),
        None if Xc is None else Xc.ctypes.data_as(ctypes.c_void_p),
        None if Wc is None else Wc.ctypes.data_as(ctypes.c_void_p), threads or default_threads())


# ---- the sumcheck that links zkAttn's tensors --------------------------------

def zkattn_link_prove(seed, Zp, X_list, Y, Yk_list, yhat, bases, rows, cols, threads=None):
    """Zp, Y: (rows*cols, 32) bytes; X_list, Yk_list: K such arrays; yhat: (rows, 32);
    bases: (K, 32).  Returns (rc, proof, point)."""
    Zp, Y, yhat, bases = [_c(a).reshape(-1, 32) for a in (Zp, Y, yhat, bases)]
    X_list = [_c(a).reshape(-1, 32) for a in X_list]
    Yk_list = [_c(a).reshape(-1, 32) for a in Yk_list]
    K = len(X_list)
    n = max(int(rows * cols).bit_length() - 1, 0)
    cap = int(lib().oracle_link_proof_bytes(_u64(rows), _u64(cols), _u64(K)))
    proof = np.zeros(cap, dtype=np.uint8)
    ln = ctypes.c_uint64(0)
    point = np.zeros((max(n, 1), 32), dtype=np.uint8)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    rc = lib().oracle_zkattn_link_prove(_p(seedb), _p(Zp), _ptr_array(X_list), _p(Y), _ptr_array(Yk_list), _p(yhat),
                                        _p(bases), _u64(rows), _u64(cols), _u64(K), _p(proof), _u64(cap),
                                        ctypes.byref(ln), _p(point), threads or default_threads())
    return rc, proof[:ln.value].tobytes() if rc == OK else b"", point[:n]


def zkattn_link_verify(seed, proof, rows, cols, bases, Zp=None, X_list=None, Y=None, Yk_list=None, yhat=None,
                       threads=None):
    bases = _c(bases).reshape(-1, 32)
    K = bases.shape[0]
    pb = np.frombuffer(bytes(proof), dtype=np.uint8).copy() if len(proof) else np.zeros(1, dtype=np.uint8)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    keep_x = [None] * K if X_list is None else [None if a is None else _c(a).reshape(-1, 32) for a in X_list]
    keep_y = [None] * K if Yk_list is None else [None if a is None else _c(a).reshape(-1, 32) for a in Yk_list]
    return lib().oracle_zkattn_link_verify(
        _p(seedb), _p(pb), _u64(len(proof)), _u64(rows), _u64(cols), _u64(K), _p(bases),
        _p(None if Zp is None else _c(Zp).reshape(-1, 32)), _ptr_array(keep_x),
        _p(None if Y is None else _c(Y).reshape(-1, 32)), _ptr_array(keep_y),
        _p(None if yhat is None else _c(yhat).reshape(-1, 32)), None, threads or default_threads())


def zkattn_link_verify_point(seed, proof, rows, cols, bases, threads=None):
    """The oracle's verifier without tensors; returns (rc, the sumcheck point v as canonical bytes)."""
    bases = _c(bases).reshape(-1, 32)
    K = bases.shape[0]
    n = max((rows * cols).bit_length() - 1, 0)
    pb = np.frombuffer(bytes(proof), dtype=np.uint8).copy() if len(proof) else np.zeros(1, dtype=np.uint8)
    seedb = _c(np.frombuffer(bytes(seed), dtype=np.uint8))
    point = np.zeros((max(n, 1), 32), dtype=np.uint8)
    none = [None] * K
    rc = lib().oracle_zkattn_link_verify(
        _p(seedb), _p(pb), _u64(len(proof)), _u64(rows), _u64(cols), _u64(K), _p(bases), None, _ptr_array(none), None,
        _ptr_array(none), None, _p(point), threads or default_threads())
    return rc, point[:n]
