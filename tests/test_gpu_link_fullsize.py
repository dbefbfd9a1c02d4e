"""The sumcheck that closes zkAttn-Prove (Protocol 2, last step) at the sizes its
timings are quoted for.

At 2^11 x 2^11 scores (2^22 entries per tensor, well past the shapes of
test_gpu_link.py) the oracle's prover still fits memory: the device proof, from
field vectors and from integer tensors, must equal it byte for byte.

At the full attention workload (2^17 x 2048 = 2^28 entries per tensor, six
tensors) the oracle's prover does not fit; there the oracle's verifier, which
needs no tensors, replays the device proof (every round, the final identity),
both device paths must give the same bytes, and each of the 2K + 2 values the proof
states at the final point is recomputed from its input tensor by the library's
multilinear evaluation (a code path of its own, compared with the oracle
elsewhere) at the point the oracle's verifier derived."""
import numpy as np
import pytest
import torch

import paper_2404_16109_amd as zk
from paper_2404_16109_amd import synth
from tests.gpu_common import link_tensors

pytestmark = pytest.mark.gpu
R = synth.BLS12_381_R


def _both_proofs(cfg, tensors):
    Zp, X, Y, Yk, yhat, ints = tensors
    rows, cols = cfg["rows"], cfg["cols"]
    rc, proof = zk.zkattn_link_prove(cfg["seed"], Zp, X, Y, Yk, yhat, cfg["bases"], rows, cols)
    assert rc == zk.ZK_OK
    rc, small = zk.zkattn_link_prove_small(cfg["seed"], ints["Zp"], ints["X"], ints["Y"], ints["Yk"], yhat, cfg["bases"],
                                           rows, cols)
    assert rc == zk.ZK_OK and small == proof
    return proof


def test_oracle_prover_at_2_pow_22(orc):
    cfg = synth.attention_link(heads=1, rows=1 << 11)
    rows, cols = cfg["rows"], cfg["cols"]
    assert rows * cols == 1 << 22
    tensors = link_tensors(cfg)
    proof = _both_proofs(cfg, tensors)
    ints = tensors[5]
    to = lambda t: orc.fr_from_i64(t.cpu().numpy().astype(np.int64))
    yhat_bytes = np.zeros((rows, 32), dtype=np.uint8)
    yhat_bytes[:, :8] = ints["yhat"].astype("<u8").view(np.uint8).reshape(rows, 8)
    rc, want, _ = orc.zkattn_link_prove(cfg["seed"], to(ints["Zp"]), [to(x) for x in ints["X"]], to(ints["Y"]),
                                        [to(y) for y in ints["Yk"]], yhat_bytes, orc.to_bytes(cfg["bases"]), rows, cols)
    assert rc == 0 and proof == want


def test_full_attention_workload(orc):
    cfg = synth.attention_link()
    rows, cols, K = cfg["rows"], cfg["cols"], 2
    assert (rows, cols) == (1 << 17, 2048)
    tensors = link_tensors(cfg)
    Zp, X, Y, Yk, yhat, ints = tensors
    proof = _both_proofs(cfg, tensors)
    # the oracle's verifier: rounds, final identity, the point
    rc, point = orc.zkattn_link_verify_point(cfg["seed"], proof, rows, cols, orc.to_bytes(cfg["bases"]))
    assert rc == 0
    v = orc.to_ints(point)
    assert len(v) == 28
    # the stated values Z'(v) X^(0..K-1)(v) Y(v) Y^(0..K-1)(v) close the proof; each from its tensor
    stated = [int.from_bytes(proof[len(proof) - 32 * (2 * K + 2 - q):][:32], "little") for q in range(2 * K + 2)]
    ws = torch.empty(zk.raw().fr_mle_eval_workspace_bytes(28), dtype=torch.uint8, device="cuda")
    for want, tensor in zip(stated, [Zp] + X + [Y] + Yk):
        rc, got = zk.fr_mle_eval(tensor, v, ws=ws)
        assert rc == 0 and got == want
    # and the row-sum claim at the head of the proof: yhat at the row part of the random point, which the device
    # verifier recomputes from yhat itself
    rc, claims = zk.zkattn_link_verify(cfg["seed"], proof, rows, cols, cfg["bases"], yhat=yhat)
    assert rc == zk.ZK_OK and claims["v"] == v
