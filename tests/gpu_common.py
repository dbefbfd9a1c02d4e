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
