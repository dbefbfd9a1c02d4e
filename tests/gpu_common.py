"""Helpers shared by the GPU parity tests: the same synthetic workload handed to
the oracle (numpy, canonical bytes) and to the device library (limb-major
Montgomery vectors)."""
import numpy as np
import torch

import paper_2404_16109_amd as zk
from paper_2404_16109_amd import synth


def oracle_table_and_tensor(orc, cfg):
    """(S bytes, T bytes) for the oracle from a synth config."""
    T = orc.fr_from_i64(cfg["tx"])
    if cfg["ty"] is not None:
        rho = orc.to_bytes([synth.pair_combiner(cfg["seed"])])[0]
        T = orc.fr_axpy(T, rho, orc.fr_from_i64(cfg["ty"]))
    S = T[cfg["idx"].astype(np.int64)]
    return S, T


def device_table_and_tensor(cfg):
    """(S Vec, T Vec, idx tensor) on the GPU from a synth config, using the
    library's own embedding and pair combination."""
    N, D = cfg["N"], cfg["D"]
    T = zk.Vec(N)
    tx = torch.from_numpy(cfg["tx"].astype(np.int32)).cuda()
    assert zk.fr_from_i32(T, tx) == zk.ZK_OK
    if cfg["ty"] is not None:
        Y = zk.Vec(N)
        ty = torch.from_numpy(cfg["ty"].astype(np.int32)).cuda()
        assert zk.fr_from_i32(Y, ty) == zk.ZK_OK
        assert zk.fr_axpy(T, T, synth.pair_combiner(cfg["seed"]), Y) == zk.ZK_OK
    idx = torch.from_numpy(cfg["idx"].astype(np.int32)).cuda()
    S = zk.Vec(D)
    S.data.copy_(T.data[:, :N].index_select(1, idx.long()))
    return S, T, idx


def first_difference(a, b):
    """Byte offset of the first difference between two byte strings, or -1."""
    if a == b:
        return -1
    n = min(len(a), len(b))
    for i in range(n):
        if a[i] != b[i]:
            return i
    return n


def link_tensors(cfg):
    """The tensors of zkAttn's closing sumcheck for a synth.attention_link config, on
    the GPU: digits X^(k), segment outputs Y^(k) = table_k[X^(k)], Y = Y^(0) Y^(1),
    Z' = -(X^(0) + 2^16 X^(1)) and the row sums yhat, as field vectors (built with
    the library's elementwise calls) and as the integers they are (for the integer
    entry point).  Returns (Zp, X, Y, Yk, yhat, ints)."""
    rows, cols = cfg["rows"], cfg["cols"]
    D = rows * cols
    X, Yk = [], []
    ints = {"X": [], "Yk": []}
    yprod = None
    for k in range(2):
        xi = torch.from_numpy(cfg["x"][k].astype(np.int32)).cuda()
        xv = zk.Vec(D)
        assert zk.fr_from_i32(xv, xi) == 0
        X.append(xv)
        yi = torch.from_numpy(cfg["ty"][k].astype(np.int32)).cuda()[xi.long()]
        yv = zk.Vec(D)
        assert zk.fr_from_i32(yv, yi) == 0
        Yk.append(yv)
        yprod = yi.long() if yprod is None else yprod * yi.long()
        ints["X"].append(xi)
        ints["Yk"].append(yi)
    yhat_int = yprod.reshape(rows, cols).sum(dim=1).cpu().numpy().astype(np.uint64)
    ints["Y"] = yprod
    Y = zk.Vec(D)
    assert zk.fr_mul(Y, Yk[0], Yk[1]) == 0
    Zp = zk.Vec(D)
    assert zk.fr_axpy(Zp, X[0], cfg["bases"][1], X[1]) == 0
    assert zk.fr_mul_scalar(Zp, Zp, synth.BLS12_381_R - 1) == 0
    canon = np.zeros((rows, 32), dtype=np.uint8)
    canon[:, :8] = yhat_int.astype("<u8").view(np.uint8).reshape(rows, 8)
    yhat = zk.vec_from_bytes(canon)
    ints["Zp"] = -(ints["X"][0].long() + cfg["bases"][1] * ints["X"][1].long())
    ints["yhat"] = yhat_int
    return Zp, X, Y, Yk, yhat, ints
