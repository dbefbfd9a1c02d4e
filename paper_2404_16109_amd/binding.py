"""ctypes binding of the C boundary declared in ``include/zkmi.h``.

Every function here has the name of the C entry point it calls and does
nothing but marshal arguments: device buffers are torch tensors (int32 storage
standing for uint32 limbs), host scalars are Python ints in [0, r).
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libzkmi.so")

ZK_OK, ZK_E_BADARG, ZK_E_NOT_IN_TABLE, ZK_E_ZERO_DENOM, ZK_E_REJECT, ZK_E_BUFSZ, ZK_E_HIP = 0, -1, -2, -3, -4, -5, -6


class fr_t(ctypes.Structure):
    _fields_ = [("l", ctypes.c_uint32 * 8)]


class fr_vec(ctypes.Structure):
    _fields_ = [("limbs", ctypes.c_void_p), ("n", ctypes.c_size_t), ("stride", ctypes.c_size_t)]


class tlookup_aux(ctypes.Structure):
    _fields_ = [("beta", fr_t), ("alpha", fr_t), ("sum_A", fr_t), ("sum_mB", fr_t), ("bad_index", ctypes.c_uint64)]


class tlookup_witness(ctypes.Structure):
    _fields_ = [("S", fr_vec), ("A", fr_vec), ("B", fr_vec), ("m", ctypes.c_void_p)]


class tlookup_claims(ctypes.Structure):
    _fields_ = [("A_v", fr_t), ("S_v", fr_t), ("B_vp", fr_t), ("m_vp", fr_t), ("T_vp", fr_t), ("v", fr_t * 32),
                ("nvars", ctypes.c_int)]


TLOOKUP_BATCH_MAX = 8
ZKATTN_LINK_MAX_K = 3


class tlookup_batch_aux(ctypes.Structure):
    _fields_ = [("beta", fr_t), ("alpha", fr_t), ("lambda_", fr_t), ("sum_A", fr_t * TLOOKUP_BATCH_MAX),
                ("sum_mB", fr_t * TLOOKUP_BATCH_MAX), ("bad_instance", ctypes.c_uint64), ("bad_index", ctypes.c_uint64)]


class tlookup_batch_claims(ctypes.Structure):
    _fields_ = [("value", (fr_t * 5) * TLOOKUP_BATCH_MAX), ("v", fr_t * 32), ("lambda_", fr_t),
                ("nvars", ctypes.c_int), ("count", ctypes.c_int)]


class zkattn_link_witness(ctypes.Structure):
    _fields_ = [("Zp", fr_vec), ("Y", fr_vec), ("yhat", fr_vec), ("X", fr_vec * ZKATTN_LINK_MAX_K),
                ("Yk", fr_vec * ZKATTN_LINK_MAX_K)]


class zkattn_link_claims(ctypes.Structure):
    _fields_ = [("yhat_u", fr_t), ("Zp_v", fr_t), ("Y_v", fr_t), ("X_v", fr_t * ZKATTN_LINK_MAX_K),
                ("Yk_v", fr_t * ZKATTN_LINK_MAX_K), ("u", fr_t * 32), ("v", fr_t * 32), ("nvars", ctypes.c_int),
                ("K", ctypes.c_int)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libzkmi.so is not built (expected at %s); run `python -m paper_2404_16109_amd.build`. "
            "There is no fallback implementation." % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    sz, vp, i32 = ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int
    P = ctypes.POINTER
    sigs = {
        "zkmi_version": (i32, []),
        "zkmi_sha256": (i32, [ctypes.c_char_p, sz, ctypes.c_char_p, i32]),
        "zkmi_selftest_resident_wait": (i32, [vp, sz, vp]),
        "zkmi_selftest_tlookup_plan": (i32, [sz, sz, sz, i32, P(ctypes.c_int32), sz]),
        "zkmi_selftest_host_rounds": (i32, [P(fr_t)] * 5 + [sz, sz, P(fr_t), P(fr_t), P(fr_t), P(fr_t), P(fr_t)]),
        "zkmi_profile_enable": (i32, [i32]),
        "zkmi_profile_reset": (i32, []),
        "zkmi_profile_query": (i32, [ctypes.c_char_p, P(ctypes.c_uint64), P(ctypes.c_double)]),
        "fr_constants": (i32, [P(fr_t), P(fr_t), P(fr_t), P(ctypes.c_uint32)]),
        "fr_from_i32": (i32, [fr_vec, vp, sz, vp]),
        "fr_from_canonical": (i32, [fr_vec, vp, sz, vp]),
        "fr_to_canonical": (i32, [vp, fr_vec, sz, vp]),
        "fr_add": (i32, [fr_vec, fr_vec, fr_vec, vp]),
        "fr_sub": (i32, [fr_vec, fr_vec, fr_vec, vp]),
        "fr_mul": (i32, [fr_vec, fr_vec, fr_vec, vp]),
        "fr_add_scalar": (i32, [fr_vec, fr_vec, P(fr_t), vp]),
        "fr_mul_scalar": (i32, [fr_vec, fr_vec, P(fr_t), vp]),
        "fr_axpy": (i32, [fr_vec, fr_vec, P(fr_t), fr_vec, vp]),
        "fr_batch_inverse_workspace_bytes": (sz, [sz]),
        "fr_batch_inverse": (i32, [fr_vec, fr_vec, vp, sz, vp]),
        "fr_sum_workspace_bytes": (sz, [sz]),
        "fr_sum": (i32, [P(fr_t), fr_vec, vp, sz, vp]),
        "fr_sum_noalloc": (i32, [vp, fr_vec, vp]),
        "fr_eq_table": (i32, [fr_vec, P(fr_t), i32, vp]),
        "fr_mle_eval_workspace_bytes": (sz, [i32]),
        "fr_mle_eval": (i32, [P(fr_t), fr_vec, P(fr_t), i32, vp, sz, vp]),
        "tlookup_workspace_bytes": (sz, [sz, sz]),
        "tlookup_multiplicities": (i32, [vp, fr_vec, vp, fr_vec, vp, sz, P(ctypes.c_uint64), vp]),
        "zkmi_thread_init": (i32, [sz]),
        "zkmi_thread_release": (i32, []),
        "tlookup_proof_bytes": (sz, [sz]),
        "tlookup_prove": (i32, [vp, fr_vec, vp, fr_vec, vp, sz, P(sz), P(tlookup_aux), vp, sz, vp]),
        "tlookup_prove_by_rows": (i32, [vp, fr_vec, vp, fr_vec, vp, sz, P(sz), P(tlookup_aux), vp, sz, vp]),
        "tlookup_prove_checked": (i32, [vp, fr_vec, vp, fr_vec, vp, sz, P(sz), P(tlookup_aux), vp, sz, vp]),
        "tlookup_small_workspace_bytes": (sz, [sz, sz]),
        "tlookup_prove_small": (i32, [vp, vp, vp, P(fr_t), sz, vp, fr_vec, vp, sz, P(sz), P(tlookup_aux), vp, sz, vp]),
        "tlookup_prove_with_beta": (i32, [vp, fr_vec, vp, fr_vec, P(fr_t), vp, sz, P(sz), P(tlookup_aux), vp, sz, vp]),
        "tlookup_verify_workspace_bytes": (sz, [sz, sz]),
        "tlookup_verify": (i32, [vp, vp, sz, fr_vec, sz, P(tlookup_witness), P(tlookup_claims), vp, sz, vp]),
        "tlookup_batch_proof_bytes": (sz, [sz, sz]),
        "tlookup_batch_workspace_bytes": (sz, [sz, sz, sz]),
        "tlookup_prove_batch": (i32, [vp, P(fr_vec), P(vp), P(fr_vec), sz, vp, sz, P(sz), P(tlookup_batch_aux), vp, sz,
                                      vp]),
        "tlookup_verify_batch": (i32, [vp, vp, sz, P(fr_vec), sz, sz, P(tlookup_witness), P(tlookup_batch_claims), vp,
                                       sz, vp]),
        "tlookup_multi_proof_bytes": (sz, [P(sz), sz]),
        "tlookup_multi_workspace_bytes": (sz, [P(sz), P(sz), sz]),
        "tlookup_prove_multi": (i32, [vp, P(fr_vec), P(vp), P(fr_vec), sz, vp, sz, P(sz), P(tlookup_batch_aux), vp, sz,
                                      vp]),
        "tlookup_multi_verify_workspace_bytes": (sz, [P(sz), P(sz), sz]),
        "tlookup_verify_multi": (i32, [vp, vp, sz, P(fr_vec), P(sz), sz, P(tlookup_witness), P(tlookup_batch_claims), vp,
                                       sz, vp]),
        "sumcheck_product_proof_bytes": (sz, [sz]),
        "sumcheck_product_workspace_bytes": (sz, [sz]),
        "sumcheck_prove_product": (i32, [vp, fr_vec, fr_vec, P(fr_t), vp, sz, P(sz), vp, sz, vp]),
        "sumcheck_verify_product": (i32, [vp, vp, sz, sz, P(fr_t), P(fr_t)]),
        "matmul_proof_bytes": (sz, [sz]),
        "matmul_workspace_bytes": (sz, [sz, sz, sz]),
        "matmul_sumcheck_prove": (i32, [vp, fr_vec, sz, sz, fr_vec, sz, vp, sz, P(sz), vp, sz, vp]),
        "matmul_sumcheck_prove_i16": (i32, [vp, vp, sz, sz, vp, sz, vp, sz, P(sz), vp, sz, vp]),
        "matmul_verify_workspace_bytes": (sz, [sz, sz, sz]),
        "matmul_sumcheck_verify": (i32, [vp, vp, sz, sz, sz, sz, fr_vec, fr_vec, fr_vec, vp, sz, vp]),
        "zkattn_link_proof_bytes": (sz, [sz, sz, sz]),
        "zkattn_link_workspace_bytes": (sz, [sz, sz, sz]),
        "zkattn_link_prove_small": (i32, [vp, vp, P(vp), vp, P(vp), fr_vec, P(ctypes.c_uint64), sz, sz, sz, vp, sz, P(sz),
                                          vp, sz, vp]),
        "zkattn_link_prove": (i32, [vp, fr_vec, P(fr_vec), fr_vec, P(fr_vec), fr_vec, P(fr_t), sz, sz, sz, vp, sz, P(sz),
                                    vp, sz, vp]),
        "zkattn_link_verify_workspace_bytes": (sz, [sz, sz]),
        "zkattn_link_verify": (i32, [vp, vp, sz, sz, sz, sz, P(fr_t), P(zkattn_link_witness), P(zkattn_link_claims), vp,
                                     sz, vp]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


_lib = _load()
EXPORTS = ["zkmi_version", "zkmi_thread_init", "zkmi_thread_release", "zkmi_sha256", "zkmi_selftest_resident_wait", "zkmi_selftest_tlookup_plan", "zkmi_selftest_host_rounds", "zkmi_profile_enable", "zkmi_profile_reset", "zkmi_profile_query", "fr_constants", "fr_from_i32", "fr_from_canonical", "fr_to_canonical", "fr_add", "fr_sub",
           "fr_mul", "fr_add_scalar", "fr_mul_scalar", "fr_axpy", "fr_batch_inverse_workspace_bytes",
           "fr_batch_inverse", "fr_sum_workspace_bytes", "fr_sum", "fr_sum_noalloc", "fr_eq_table", "fr_mle_eval_workspace_bytes",
           "fr_mle_eval", "tlookup_workspace_bytes", "tlookup_multiplicities", "tlookup_proof_bytes", "tlookup_prove",
           "tlookup_prove_by_rows", "tlookup_prove_checked", "tlookup_small_workspace_bytes", "tlookup_prove_small", "tlookup_prove_with_beta", "tlookup_verify_workspace_bytes", "tlookup_verify",
           "tlookup_batch_proof_bytes", "tlookup_batch_workspace_bytes", "tlookup_prove_batch", "tlookup_verify_batch",
           "tlookup_multi_proof_bytes", "tlookup_multi_workspace_bytes", "tlookup_prove_multi",
           "tlookup_multi_verify_workspace_bytes", "tlookup_verify_multi",
           "sumcheck_product_proof_bytes", "sumcheck_product_workspace_bytes", "sumcheck_prove_product",
           "sumcheck_verify_product", "matmul_proof_bytes", "matmul_workspace_bytes", "matmul_sumcheck_prove", "matmul_sumcheck_prove_i16",
           "matmul_verify_workspace_bytes", "matmul_sumcheck_verify", "zkattn_link_proof_bytes",
           "zkattn_link_workspace_bytes", "zkattn_link_prove", "zkattn_link_prove_small",
           "zkattn_link_verify_workspace_bytes",
           "zkattn_link_verify"]


def raw():
    """The ctypes library handle."""
    return _lib


# ---- marshalling helpers ------------------------------------------------------------

def _fr(x):
    out = fr_t()
    x = int(x)
    for k in range(8):
        out.l[k] = (x >> (32 * k)) & 0xFFFFFFFF
    return out


def _fr_int(f):
    return sum(int(f.l[k]) << (32 * k) for k in range(8))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _seed(seed):
    seed = bytes(seed)
    assert len(seed) == 32
    return ctypes.create_string_buffer(seed, 32)


class Vec:
    """A device vector of n field elements: int32 tensor of shape (8, stride)."""

    def __init__(self, n, stride=None, device="cuda"):
        self.n = int(n)
        self.stride = int(stride if stride is not None else max(n, 1))
        self.data = torch.empty((8, self.stride), dtype=torch.int32, device=device)

    @property
    def c(self):
        return fr_vec(self.data.data_ptr(), self.n, self.stride)


_EMPTY = fr_vec(None, 0, 0)


def _ws(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


# ---- field library ----------------------------------------------------------------------

def zkmi_version():
    return _lib.zkmi_version()


def zkmi_sha256(data, use_sha_instructions=True):
    """(used_instruction_path, digest) of host bytes."""
    out = ctypes.create_string_buffer(32)
    buf = bytes(data)
    rc = _lib.zkmi_sha256(buf, len(buf), out, 1 if use_sha_instructions else 0)
    return rc, out.raw


def zkmi_selftest_resident_wait():
    ws = _ws(4096)
    return _lib.zkmi_selftest_resident_wait(ws.data_ptr(), ws.numel(), _stream())


def zkmi_selftest_tlookup_plan(D, N, K=1, from_ints=False):
    """Returns (rc, list of (kernel, s_source, in32, out32) per round); runs on the host only."""
    out = (ctypes.c_int32 * (4 * 32))()
    rc = _lib.zkmi_selftest_tlookup_plan(D, N, K, 1 if from_ints else 0, out, 32)
    rounds = [tuple(out[4 * k:4 * k + 4]) for k in range(max(rc, 0))]
    return rc, rounds


def zkmi_selftest_host_rounds(A, S, B, M, T, u_rest, beta, challenges):
    """The host's rounds on lists of integers; returns (rc, sums: 11 per round, finals: 5); runs on the host only."""
    def arr(xs):
        out = (fr_t * max(len(xs), 1))()
        for i, x in enumerate(xs):
            out[i] = _fr(x)
        return out
    rounds = max(len(A).bit_length() - 1, 1)
    sums = (fr_t * (11 * rounds))()
    finals = (fr_t * 5)()
    rc = _lib.zkmi_selftest_host_rounds(arr(A), arr(S), arr(B), arr(M), arr(T), len(A), len(B), arr(u_rest), _fr(beta),
                                        arr(challenges), sums, finals)
    return rc, [_fr_int(x) for x in sums], [_fr_int(x) for x in finals]


def zkmi_thread_init(max_table_rows):
    return _lib.zkmi_thread_init(max_table_rows)


def zkmi_thread_release():
    return _lib.zkmi_thread_release()


def zkmi_profile_enable(on):
    return _lib.zkmi_profile_enable(1 if on else 0)


def zkmi_profile_reset():
    return _lib.zkmi_profile_reset()


def zkmi_profile_query(phase):
    """Returns (rc, records, total_ms)."""
    n, ms = ctypes.c_uint64(0), ctypes.c_double(0.0)
    rc = _lib.zkmi_profile_query(phase.encode(), ctypes.byref(n), ctypes.byref(ms))
    return rc, n.value, ms.value


def fr_constants():
    m, r1, r2, ninv = fr_t(), fr_t(), fr_t(), ctypes.c_uint32(0)
    rc = _lib.fr_constants(ctypes.byref(m), ctypes.byref(r1), ctypes.byref(r2), ctypes.byref(ninv))
    return rc, _fr_int(m), _fr_int(r1), _fr_int(r2), ninv.value


def fr_from_i32(dst, src):
    assert src.dtype == torch.int32 and src.is_cuda and src.is_contiguous()
    return _lib.fr_from_i32(dst.c, src.data_ptr(), src.numel(), _stream())


def fr_from_canonical(dst, aos):
    """aos: int32/uint8 cuda tensor holding n x 32 bytes (canonical little-endian)."""
    assert aos.is_cuda and aos.is_contiguous() and aos.numel() * aos.element_size() == 32 * dst.n
    return _lib.fr_from_canonical(dst.c, aos.data_ptr(), dst.n, _stream())


def fr_to_canonical(aos, src):
    assert aos.is_cuda and aos.is_contiguous() and aos.numel() * aos.element_size() == 32 * src.n
    return _lib.fr_to_canonical(aos.data_ptr(), src.c, src.n, _stream())


def fr_add(dst, a, b):
    return _lib.fr_add(dst.c, a.c, b.c, _stream())


def fr_sub(dst, a, b):
    return _lib.fr_sub(dst.c, a.c, b.c, _stream())


def fr_mul(dst, a, b):
    return _lib.fr_mul(dst.c, a.c, b.c, _stream())


def fr_add_scalar(dst, x, s):
    return _lib.fr_add_scalar(dst.c, x.c, ctypes.byref(_fr(s)), _stream())


def fr_mul_scalar(dst, x, s):
    return _lib.fr_mul_scalar(dst.c, x.c, ctypes.byref(_fr(s)), _stream())


def fr_axpy(dst, x, s, y):
    return _lib.fr_axpy(dst.c, x.c, ctypes.byref(_fr(s)), y.c, _stream())


def fr_batch_inverse_workspace_bytes(n):
    return _lib.fr_batch_inverse_workspace_bytes(n)


def fr_batch_inverse(dst, src, ws=None):
    ws = ws if ws is not None else _ws(fr_batch_inverse_workspace_bytes(src.n))
    return _lib.fr_batch_inverse(dst.c, src.c, ws.data_ptr(), ws.numel(), _stream())


def fr_sum(a, ws=None):
    ws = ws if ws is not None else _ws(_lib.fr_sum_workspace_bytes(a.n))
    out = fr_t()
    rc = _lib.fr_sum(ctypes.byref(out), a.c, ws.data_ptr(), ws.numel(), _stream())
    return rc, _fr_int(out)


def fr_sum_noalloc(out, a):
    """out: int32 cuda tensor of 8 words, written when the current stream gets there."""
    assert out.is_cuda and out.is_contiguous() and out.numel() * out.element_size() == 32
    return _lib.fr_sum_noalloc(out.data_ptr(), a.c, _stream())


def fr_eq_table(dst, u):
    arr = (fr_t * max(len(u), 1))(*[_fr(x) for x in u])
    return _lib.fr_eq_table(dst.c, arr, len(u), _stream())


def fr_mle_eval(a, point, ws=None):
    nv = len(point)
    ws = ws if ws is not None else _ws(_lib.fr_mle_eval_workspace_bytes(nv))
    arr = (fr_t * max(nv, 1))(*[_fr(x) for x in point])
    out = fr_t()
    rc = _lib.fr_mle_eval(ctypes.byref(out), a.c, arr, nv, ws.data_ptr(), ws.numel(), _stream())
    return rc, _fr_int(out)


# ---- tlookup -------------------------------------------------------------------------------

def tlookup_workspace_bytes(D, N):
    return _lib.tlookup_workspace_bytes(D, N)


def tlookup_proof_bytes(D):
    return _lib.tlookup_proof_bytes(D)


def _idx_ptr(idx):
    if idx is None:
        return None
    assert idx.is_cuda and idx.is_contiguous() and idx.element_size() == 4
    return idx.data_ptr()


def tlookup_multiplicities(S, idx, T, ws=None):
    """Returns (rc, m as an int32 cuda tensor of N counts, bad_index)."""
    ws = ws if ws is not None else _ws(tlookup_workspace_bytes(S.n, T.n))
    m = torch.empty(max(T.n, 1), dtype=torch.int32, device="cuda")
    bad = ctypes.c_uint64(0)
    rc = _lib.tlookup_multiplicities(m.data_ptr(), S.c, _idx_ptr(idx), T.c, ws.data_ptr(), ws.numel(),
                                     ctypes.byref(bad), _stream())
    return rc, m, bad.value


def _aux_dict(aux):
    return {"beta": _fr_int(aux.beta), "alpha": _fr_int(aux.alpha), "sum_A": _fr_int(aux.sum_A),
            "sum_mB": _fr_int(aux.sum_mB), "bad_index": int(aux.bad_index)}


def tlookup_prove_by_rows(seed, S, idx, T, ws=None, cap=None):
    """Returns (rc, proof bytes, aux dict with 'len')."""
    ws = ws if ws is not None else _ws(tlookup_workspace_bytes(S.n, T.n))
    cap = tlookup_proof_bytes(S.n) if cap is None else cap
    proof = ctypes.create_string_buffer(max(cap, 1))
    ln = ctypes.c_size_t(0)
    aux = tlookup_aux()
    rc = _lib.tlookup_prove_by_rows(_seed(seed), S.c, _idx_ptr(idx), T.c, proof, cap, ctypes.byref(ln), ctypes.byref(aux),
                                    ws.data_ptr(), ws.numel(), _stream())
    info = _aux_dict(aux)
    info["len"] = ln.value
    return rc, proof.raw[:ln.value] if rc == ZK_OK else b"", info


def tlookup_prove_checked(seed, S, idx, T, ws=None, cap=None):
    """Returns (rc, proof bytes, aux dict with 'len')."""
    ws = ws if ws is not None else _ws(tlookup_workspace_bytes(S.n, T.n))
    cap = tlookup_proof_bytes(S.n) if cap is None else cap
    proof = ctypes.create_string_buffer(max(cap, 1))
    ln = ctypes.c_size_t(0)
    aux = tlookup_aux()
    rc = _lib.tlookup_prove_checked(_seed(seed), S.c, _idx_ptr(idx), T.c, proof, cap, ctypes.byref(ln), ctypes.byref(aux),
                                    ws.data_ptr(), ws.numel(), _stream())
    info = _aux_dict(aux)
    info["len"] = ln.value
    return rc, proof.raw[:ln.value] if rc == ZK_OK else b"", info


def tlookup_prove(seed, S, idx, T, ws=None, cap=None, forced_beta=None):
    """Returns (rc, proof bytes, aux dict with 'len')."""
    ws = ws if ws is not None else _ws(tlookup_workspace_bytes(S.n, T.n))
    cap = tlookup_proof_bytes(S.n) if cap is None else cap
    proof = ctypes.create_string_buffer(max(cap, 1))
    ln = ctypes.c_size_t(0)
    aux = tlookup_aux()
    if forced_beta is None:
        rc = _lib.tlookup_prove(_seed(seed), S.c, _idx_ptr(idx), T.c, proof, cap, ctypes.byref(ln), ctypes.byref(aux),
                                ws.data_ptr(), ws.numel(), _stream())
    else:
        rc = _lib.tlookup_prove_with_beta(_seed(seed), S.c, _idx_ptr(idx), T.c, ctypes.byref(_fr(forced_beta)), proof,
                                          cap, ctypes.byref(ln), ctypes.byref(aux), ws.data_ptr(), ws.numel(),
                                          _stream())
    info = _aux_dict(aux)
    info["len"] = ln.value
    return rc, proof.raw[:ln.value] if rc == ZK_OK else b"", info


def tlookup_small_workspace_bytes(D, N):
    return _lib.tlookup_small_workspace_bytes(D, N)


def tlookup_prove_small(seed, X, Y, rho, idx, T, ws=None, cap=None):
    """X, Y: int32 device tensors of D entries (Y and rho may both be None); idx: int32 hints.
    Returns (rc, proof bytes, aux dict with 'len')."""
    D = X.numel()
    assert X.dtype == torch.int32 and X.is_contiguous() and (Y is None or (Y.dtype == torch.int32 and Y.numel() == D))
    ws = ws if ws is not None else _ws(_lib.tlookup_small_workspace_bytes(D, T.n))
    cap = tlookup_proof_bytes(D) if cap is None else cap
    proof = ctypes.create_string_buffer(max(cap, 1))
    ln = ctypes.c_size_t(0)
    aux = tlookup_aux()
    rc = _lib.tlookup_prove_small(_seed(seed), X.data_ptr(), Y.data_ptr() if Y is not None else None,
                                  ctypes.byref(_fr(rho)) if rho is not None else None, D, _idx_ptr(idx), T.c, proof, cap,
                                  ctypes.byref(ln), ctypes.byref(aux), ws.data_ptr(), ws.numel(), _stream())
    info = _aux_dict(aux)
    info["len"] = ln.value
    return rc, proof.raw[:ln.value] if rc == ZK_OK else b"", info


def tlookup_verify(seed, proof, T, D, S=None, A=None, B=None, m=None, ws=None):
    """Returns (rc, claims dict)."""
    ws = ws if ws is not None else _ws(_lib.tlookup_verify_workspace_bytes(D, T.n))
    wit = None
    if S is not None or A is not None or B is not None or m is not None:
        wit = tlookup_witness(S.c if S is not None else _EMPTY, A.c if A is not None else _EMPTY,
                              B.c if B is not None else _EMPTY, m.data_ptr() if m is not None else None)
    claims = tlookup_claims()
    pb = ctypes.create_string_buffer(bytes(proof), max(len(proof), 1))
    rc = _lib.tlookup_verify(_seed(seed), pb, len(proof), T.c, D, ctypes.byref(wit) if wit is not None else None,
                             ctypes.byref(claims), ws.data_ptr(), ws.numel(), _stream())
    out = {}
    if rc == ZK_OK:
        out = {"A_v": _fr_int(claims.A_v), "S_v": _fr_int(claims.S_v), "B_vp": _fr_int(claims.B_vp),
               "m_vp": _fr_int(claims.m_vp), "T_vp": _fr_int(claims.T_vp),
               "v": [_fr_int(claims.v[t]) for t in range(claims.nvars)]}
    return rc, out


def tlookup_batch_proof_bytes(D, K):
    return _lib.tlookup_batch_proof_bytes(D, K)


def tlookup_batch_workspace_bytes(D, N, K):
    return _lib.tlookup_batch_workspace_bytes(D, N, K)


def tlookup_prove_batch(seed, S, idx, T, ws=None, cap=None):
    """S, T: lists of K Vec; idx: None or a list of K (tensor or None).
    Returns (rc, proof bytes, aux dict with 'len')."""
    K = len(S)
    assert len(T) == K and (idx is None or len(idx) == K)
    D, N = S[0].n, T[0].n
    ws = ws if ws is not None else _ws(tlookup_batch_workspace_bytes(D, N, K))
    cap = tlookup_batch_proof_bytes(D, K) if cap is None else cap
    proof = ctypes.create_string_buffer(max(cap, 1))
    ln = ctypes.c_size_t(0)
    aux = tlookup_batch_aux()
    Sv = (fr_vec * K)(*[s.c for s in S])
    Tv = (fr_vec * K)(*[t.c for t in T])
    Iv = None
    if idx is not None:
        Iv = (ctypes.c_void_p * K)(*[_idx_ptr(i) for i in idx])
    rc = _lib.tlookup_prove_batch(_seed(seed), Sv, Iv, Tv, K, proof, cap, ctypes.byref(ln), ctypes.byref(aux),
                                  ws.data_ptr(), ws.numel(), _stream())
    info = {"beta": _fr_int(aux.beta), "alpha": _fr_int(aux.alpha), "lambda": _fr_int(aux.lambda_),
            "sum_A": [_fr_int(aux.sum_A[i]) for i in range(min(K, TLOOKUP_BATCH_MAX))],
            "sum_mB": [_fr_int(aux.sum_mB[i]) for i in range(min(K, TLOOKUP_BATCH_MAX))],
            "bad_instance": int(aux.bad_instance), "bad_index": int(aux.bad_index), "len": ln.value}
    return rc, proof.raw[:ln.value] if rc == ZK_OK else b"", info


def tlookup_verify_batch(seed, proof, T, D, S=None, A=None, B=None, m=None, ws=None):
    """T: list of K Vec; S, A, B, m: None or lists of K (entries may be None).
    Returns (rc, claims dict)."""
    K = len(T)
    ws = ws if ws is not None else _ws(_lib.tlookup_verify_workspace_bytes(D, T[0].n))
    Tv = (fr_vec * K)(*[t.c for t in T])
    wit = None
    if any(x is not None for x in (S, A, B, m)):
        def member(lst, i):
            return lst[i].c if lst is not None and lst[i] is not None else _EMPTY
        wit = (tlookup_witness * K)(*[
            tlookup_witness(member(S, i), member(A, i), member(B, i),
                            m[i].data_ptr() if m is not None and m[i] is not None else None) for i in range(K)])
    claims = tlookup_batch_claims()
    pb = ctypes.create_string_buffer(bytes(proof), max(len(proof), 1))
    rc = _lib.tlookup_verify_batch(_seed(seed), pb, len(proof), Tv, K, D, wit, ctypes.byref(claims), ws.data_ptr(),
                                   ws.numel(), _stream())
    out = {}
    if rc == ZK_OK:
        out = {"lambda": _fr_int(claims.lambda_), "v": [_fr_int(claims.v[t]) for t in range(claims.nvars)],
               "value": [[_fr_int(claims.value[i][q]) for q in range(5)] for i in range(K)]}
    return rc, out


def _sizes(values):
    return (ctypes.c_size_t * len(values))(*[int(v) for v in values])


def tlookup_multi_proof_bytes(Ds):
    return _lib.tlookup_multi_proof_bytes(_sizes(Ds), len(Ds))


def tlookup_multi_workspace_bytes(Ds, Ns):
    return _lib.tlookup_multi_workspace_bytes(_sizes(Ds), _sizes(Ns), len(Ds))


def tlookup_prove_multi(seed, S, idx, T, ws=None, cap=None):
    """Lookups of any shapes under one sumcheck.  S, T: lists of K Vec (their lengths are the shapes); idx: None or a
    list of K (tensor or None).  Returns (rc, proof bytes, aux dict with 'len')."""
    K = len(S)
    assert len(T) == K and (idx is None or len(idx) == K)
    Ds, Ns = [s.n for s in S], [t.n for t in T]
    ws = ws if ws is not None else _ws(tlookup_multi_workspace_bytes(Ds, Ns))
    cap = tlookup_multi_proof_bytes(Ds) if cap is None else cap
    proof = ctypes.create_string_buffer(max(cap, 1))
    ln = ctypes.c_size_t(0)
    aux = tlookup_batch_aux()
    Sv = (fr_vec * K)(*[s.c for s in S])
    Tv = (fr_vec * K)(*[t.c for t in T])
    Iv = None
    if idx is not None:
        Iv = (ctypes.c_void_p * K)(*[_idx_ptr(i) for i in idx])
    rc = _lib.tlookup_prove_multi(_seed(seed), Sv, Iv, Tv, K, proof, cap, ctypes.byref(ln), ctypes.byref(aux),
                                  ws.data_ptr(), ws.numel(), _stream())
    info = {"beta": _fr_int(aux.beta), "alpha": _fr_int(aux.alpha), "lambda": _fr_int(aux.lambda_),
            "sum_A": [_fr_int(aux.sum_A[i]) for i in range(min(K, TLOOKUP_BATCH_MAX))],
            "sum_mB": [_fr_int(aux.sum_mB[i]) for i in range(min(K, TLOOKUP_BATCH_MAX))],
            "bad_instance": int(aux.bad_instance), "bad_index": int(aux.bad_index), "len": ln.value}
    return rc, proof.raw[:ln.value] if rc == ZK_OK else b"", info


def tlookup_verify_multi(seed, proof, T, Ds, S=None, A=None, B=None, m=None, ws=None):
    """T: list of K Vec; Ds: the K tensor lengths; S, A, B, m: None or lists of K (entries may be None).
    Returns (rc, claims dict); instance i's claims are at v[len(v) - log2 Ds[i]:]."""
    K = len(T)
    Ns = [t.n for t in T]
    ws = ws if ws is not None else _ws(_lib.tlookup_multi_verify_workspace_bytes(_sizes(Ds), _sizes(Ns), K))
    Tv = (fr_vec * K)(*[t.c for t in T])
    wit = None
    if any(x is not None for x in (S, A, B, m)):
        def member(lst, i):
            return lst[i].c if lst is not None and lst[i] is not None else _EMPTY
        wit = (tlookup_witness * K)(*[
            tlookup_witness(member(S, i), member(A, i), member(B, i),
                            m[i].data_ptr() if m is not None and m[i] is not None else None) for i in range(K)])
    claims = tlookup_batch_claims()
    pb = ctypes.create_string_buffer(bytes(proof), max(len(proof), 1))
    rc = _lib.tlookup_verify_multi(_seed(seed), pb, len(proof), Tv, _sizes(Ds), K, wit, ctypes.byref(claims),
                                   ws.data_ptr(), ws.numel(), _stream())
    out = {}
    if rc == ZK_OK:
        out = {"lambda": _fr_int(claims.lambda_), "v": [_fr_int(claims.v[t]) for t in range(claims.nvars)],
               "value": [[_fr_int(claims.value[i][q]) for q in range(5)] for i in range(K)]}
    return rc, out


# ---- product sumcheck / matmul -----------------------------------------------------------------

def sumcheck_prove_product(seed, a, b, claim, ws=None, cap=None):
    """a, b are folded in place.  Returns (rc, proof bytes)."""
    ws = ws if ws is not None else _ws(_lib.sumcheck_product_workspace_bytes(a.n))
    cap = _lib.sumcheck_product_proof_bytes(a.n) if cap is None else cap
    proof = ctypes.create_string_buffer(max(cap, 1))
    ln = ctypes.c_size_t(0)
    rc = _lib.sumcheck_prove_product(_seed(seed), a.c, b.c, ctypes.byref(_fr(claim)), proof, cap, ctypes.byref(ln),
                                     ws.data_ptr(), ws.numel(), _stream())
    return rc, proof.raw[:ln.value] if rc == ZK_OK else b""


def sumcheck_verify_product(seed, proof, n):
    """Host only.  Returns (rc, [a(r), b(r)], point)."""
    fin = (fr_t * 2)()
    pt = (fr_t * 32)()
    pb = ctypes.create_string_buffer(bytes(proof), max(len(proof), 1))
    rc = _lib.sumcheck_verify_product(_seed(seed), pb, len(proof), n, fin, pt)
    d = max(int(n).bit_length() - 1, 0)
    return rc, [_fr_int(fin[0]), _fr_int(fin[1])], [_fr_int(pt[k]) for k in range(d)]


def matmul_workspace_bytes(D0, D1, D2):
    return _lib.matmul_workspace_bytes(D0, D1, D2)


def matmul_sumcheck_prove(seed, X, D0, D1, W, D2, ws=None, cap=None):
    ws = ws if ws is not None else _ws(matmul_workspace_bytes(D0, D1, D2))
    cap = _lib.matmul_proof_bytes(D1) if cap is None else cap
    proof = ctypes.create_string_buffer(max(cap, 1))
    ln = ctypes.c_size_t(0)
    rc = _lib.matmul_sumcheck_prove(_seed(seed), X.c, D0, D1, W.c, D2, proof, cap, ctypes.byref(ln), ws.data_ptr(),
                                    ws.numel(), _stream())
    return rc, proof.raw[:ln.value] if rc == ZK_OK else b""


def matmul_sumcheck_prove_i16(seed, X, W, ws=None, cap=None):
    """X: (D0, D1) int16 device tensor, W: (D1, D2) int16 device tensor.  Returns (rc, proof bytes)."""
    assert X.dtype == torch.int16 and W.dtype == torch.int16 and X.is_contiguous() and W.is_contiguous()
    D0, D1 = X.shape
    D2 = W.shape[1]
    assert W.shape[0] == D1
    ws = ws if ws is not None else _ws(matmul_workspace_bytes(D0, D1, D2))
    cap = _lib.matmul_proof_bytes(D1) if cap is None else cap
    proof = ctypes.create_string_buffer(max(cap, 1))
    ln = ctypes.c_size_t(0)
    rc = _lib.matmul_sumcheck_prove_i16(_seed(seed), X.data_ptr(), D0, D1, W.data_ptr(), D2, proof, cap, ctypes.byref(ln),
                                        ws.data_ptr(), ws.numel(), _stream())
    return rc, proof.raw[:ln.value] if rc == ZK_OK else b""


def matmul_sumcheck_verify(seed, proof, D0, D1, D2, Y=None, X=None, W=None, ws=None):
    ws = ws if ws is not None else _ws(_lib.matmul_verify_workspace_bytes(D0, D1, D2))
    pb = ctypes.create_string_buffer(bytes(proof), max(len(proof), 1))
    return _lib.matmul_sumcheck_verify(_seed(seed), pb, len(proof), D0, D1, D2, Y.c if Y is not None else _EMPTY,
                                       X.c if X is not None else _EMPTY, W.c if W is not None else _EMPTY,
                                       ws.data_ptr(), ws.numel(), _stream())


# ---- conveniences for tests and benches (host <-> device copies, no arithmetic) ---------------

def vec_from_bytes(arr):
    """numpy uint8 (n, 32) canonical little-endian -> device Vec (through fr_from_canonical)."""
    import numpy as np
    arr = np.ascontiguousarray(arr, dtype=np.uint8).reshape(-1, 32)
    t = torch.from_numpy(arr.view(np.int32).reshape(-1, 8).copy()).cuda()
    v = Vec(arr.shape[0])
    rc = fr_from_canonical(v, t)
    assert rc == ZK_OK, rc
    return v


def vec_to_bytes(v):
    """device Vec -> numpy uint8 (n, 32) canonical little-endian (through fr_to_canonical)."""
    import numpy as np
    t = torch.empty((max(v.n, 1), 8), dtype=torch.int32, device="cuda")
    rc = _lib.fr_to_canonical(t.data_ptr(), v.c, v.n, _stream())
    assert rc == ZK_OK, rc
    torch.cuda.synchronize()
    return t.cpu().numpy()[:v.n].view(np.uint8).reshape(-1, 32)


# ---- zkAttn: the sumcheck linking an attention layer's tensors ---------------------------------------

def zkattn_link_proof_bytes(rows, cols, K):
    return _lib.zkattn_link_proof_bytes(rows, cols, K)


def zkattn_link_workspace_bytes(rows, cols, K):
    return _lib.zkattn_link_workspace_bytes(rows, cols, K)


def zkattn_link_prove(seed, Zp, X, Y, Yk, yhat, bases, rows, cols, ws=None, cap=None):
    """Zp, Y, yhat: Vec; X, Yk: lists of K Vec; bases: K integers.  Returns (rc, proof bytes)."""
    K = len(X)
    assert len(Yk) == K and len(bases) == K
    ws = ws if ws is not None else _ws(zkattn_link_workspace_bytes(rows, cols, K))
    cap = zkattn_link_proof_bytes(rows, cols, K) if cap is None else cap
    proof = ctypes.create_string_buffer(max(cap, 1))
    ln = ctypes.c_size_t(0)
    Xv = (fr_vec * K)(*[x.c for x in X])
    Yv = (fr_vec * K)(*[y.c for y in Yk])
    Bv = (fr_t * K)(*[_fr(b) for b in bases])
    rc = _lib.zkattn_link_prove(_seed(seed), Zp.c, Xv, Y.c, Yv, yhat.c, Bv, rows, cols, K, proof, cap, ctypes.byref(ln),
                                ws.data_ptr(), ws.numel(), _stream())
    return rc, proof.raw[:ln.value] if rc == ZK_OK else b""


def zkattn_link_prove_small(seed, Zp, X, Y, Yk, yhat, bases, rows, cols, ws=None, cap=None):
    """The tensors as integers on the device: Zp int64, Y int64 (read as unsigned),
    X and Yk lists of K int32 tensors (read as unsigned); yhat: Vec; bases: K
    integers below 2^32.  Returns (rc, proof bytes)."""
    K = len(X)
    assert len(Yk) == K and len(bases) == K
    assert Zp.dtype == torch.int64 and Y.dtype == torch.int64 and all(t.dtype == torch.int32 for t in list(X) + list(Yk))
    assert all(t.is_contiguous() and t.numel() >= rows * cols for t in [Zp, Y] + list(X) + list(Yk))
    ws = ws if ws is not None else _ws(zkattn_link_workspace_bytes(rows, cols, K))
    cap = zkattn_link_proof_bytes(rows, cols, K) if cap is None else cap
    proof = ctypes.create_string_buffer(max(cap, 1))
    ln = ctypes.c_size_t(0)
    Xv = (ctypes.c_void_p * K)(*[x.data_ptr() for x in X])
    Yv = (ctypes.c_void_p * K)(*[y.data_ptr() for y in Yk])
    Bv = (ctypes.c_uint64 * K)(*[int(b) for b in bases])
    rc = _lib.zkattn_link_prove_small(_seed(seed), Zp.data_ptr(), Xv, Y.data_ptr(), Yv, yhat.c, Bv, rows, cols, K, proof,
                                      cap, ctypes.byref(ln), ws.data_ptr(), ws.numel(), _stream())
    return rc, proof.raw[:ln.value] if rc == ZK_OK else b""


def zkattn_link_verify(seed, proof, rows, cols, bases, Zp=None, X=None, Y=None, Yk=None, yhat=None, ws=None):
    """Tensors (Vec, or lists of K Vec / None) stand in for the openings.  Returns (rc, claims dict)."""
    K = len(bases)
    Bv = (fr_t * K)(*[_fr(b) for b in bases])
    wit = None
    if any(t is not None for t in (Zp, X, Y, Yk, yhat)):
        wit = zkattn_link_witness()
        wit.Zp = Zp.c if Zp is not None else _EMPTY
        wit.Y = Y.c if Y is not None else _EMPTY
        wit.yhat = yhat.c if yhat is not None else _EMPTY
        for k in range(ZKATTN_LINK_MAX_K):
            wit.X[k] = X[k].c if X is not None and k < K and X[k] is not None else _EMPTY
            wit.Yk[k] = Yk[k].c if Yk is not None and k < K and Yk[k] is not None else _EMPTY
        ws = ws if ws is not None else _ws(_lib.zkattn_link_verify_workspace_bytes(rows, cols))
    claims = zkattn_link_claims()
    pb = ctypes.create_string_buffer(bytes(proof), max(len(proof), 1))
    rc = _lib.zkattn_link_verify(_seed(seed), pb, len(proof), rows, cols, K, Bv,
                                 ctypes.byref(wit) if wit is not None else None, ctypes.byref(claims),
                                 ws.data_ptr() if ws is not None else None, ws.numel() if ws is not None else 0,
                                 _stream() if wit is not None else None)
    out = {}
    if rc == ZK_OK:
        n = claims.nvars
        out = {"yhat_u": _fr_int(claims.yhat_u), "Zp_v": _fr_int(claims.Zp_v), "Y_v": _fr_int(claims.Y_v),
               "X_v": [_fr_int(claims.X_v[k]) for k in range(K)], "Yk_v": [_fr_int(claims.Yk_v[k]) for k in range(K)],
               "u": [_fr_int(claims.u[t]) for t in range(n)], "v": [_fr_int(claims.v[t]) for t in range(n)]}
    return rc, out
