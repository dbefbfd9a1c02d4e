#!/usr/bin/env python3
"""Benchmark of the tlookup prover hot path on one MI355X.

A "step" is one whole `tlookup_prove` call (multiplicities, digest of m, both
batch inversions, the digests of A and B that stand in for their commitments, eq
tables, all sumcheck rounds with folding, transcript) on
the 7B-FFN activation-table workload: D = 2^25 elements (2048 x 11008
activations padded), N = 2^16 table rows, inputs resident in HBM as limb-major
Montgomery vectors.  Prints one JSON line.

The work model behind `value` is fixed (it does not follow the
implementation): 10 field multiplications per element of S and per table row
(3 for the batched inversion, 5 to evaluate a round's sums per pair and 2 to
fold it, pairs summing to D over all rounds).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MAD_PER_S = 256 * 64 * 2.4e9      # 256 CUs x 64 lanes x 2.4 GHz, one 32-bit multiply-add per lane per clock
MADS_PER_FR_MUL = 112                   # 64 for the 8x8-limb product + 48 for the reduction (two of r's limbs need no multiplier)
ROUND_DATA_FR_MUL_PER_PAIR_EVAL = 5     # two to weight A0, A1, three products
ROUND_DATA_FR_MUL_PER_PAIR_FOLD = 4     # two arrays, two folded entries per pair
PEAK_HBM_BYTES_PER_S = 8e12             # MI355X HBM3E, published
WHOLE_PROVE_BYTES_PER_ELEMENT = 292     # hints 4 + inversion 96 + 192 (every version of A and S counted once, when a round reads it)


def fr_mul_model(D, N):
    return 10 * D + 10 * N


def first_two_rounds_share_a_pass(D, N):
    """From a vector of field elements the first pass over A and S yields the sums of the first two rounds and folds
    nothing; the first launch of k_round_data29 is then round 2, which binds two variables at once."""
    n, h = D.bit_length() - 1, (D // N).bit_length() - 1
    return h >= 3 and (D >> 3) > 256


def rounds_on_29_bits(D, N, from_ints=False):
    """The rounds the dominant kernel (k_round_data29) runs: after the first (after the first two, when those share
    a pass), before the table's variables, while more than 256 pairs remain."""
    n, h = D.bit_length() - 1, (D // N).bit_length() - 1
    first = 2 if not from_ints and first_two_rounds_share_a_pass(D, N) else 1
    return [k for k in range(first, h) if (D >> (k + 1)) > 256]


def round29_work(D, N):
    """(pairs, algorithmic field multiplications, algorithmic bytes) of all launches of k_round_data29 in one prove.
    Per pair a round folds four entries of A and four of S into two of each (4 multiplications, 12 entries of 32 B
    moved), weights two entries and forms three products: 9 multiplications.  The round that binds two variables at
    once folds sixteen entries into four (12 multiplications, 20 entries moved): 17."""
    pairs = muls = moved = 0
    for k in rounds_on_29_bits(D, N):
        p = D >> (k + 1)
        two = k == 2 and first_two_rounds_share_a_pass(D, N)
        pairs += p
        muls += p * ((12 if two else ROUND_DATA_FR_MUL_PER_PAIR_FOLD) + ROUND_DATA_FR_MUL_PER_PAIR_EVAL)
        moved += p * (20 if two else 12) * 32
    return pairs, muls, moved


def measured_traffic():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3
    counter summary, if there is one (lines `FETCH_BYTES_PER_LAUNCH=` /
    `WRITE_BYTES_PER_LAUNCH=`)."""
    path = os.path.join(ROOT, "profiles", "round_data_c3_pmc.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        for key in ("FETCH_BYTES_PER_LAUNCH", "WRITE_BYTES_PER_LAUNCH"):
            if line.startswith(key + "="):
                vals[key] = float(line.split("=", 1)[1])
    if len(vals) == 2:
        return vals["FETCH_BYTES_PER_LAUNCH"] + vals["WRITE_BYTES_PER_LAUNCH"]
    return None


def recorded_fullsize_oracle():
    """The oracle's wall time on the headline workload at full size, recorded when the
    expected proof was written (profiles/oracle_c3_fullsize.txt: lines `SECONDS=`, `CORES=`)."""
    path = os.path.join(ROOT, "profiles", "oracle_c3_fullsize.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        for key in ("SECONDS", "CORES"):
            if line.startswith(key + "="):
                vals[key] = float(line.split("=", 1)[1])
    return vals if len(vals) == 2 else None


def measured_whole_prove_traffic():
    """HBM bytes of one whole prove from the committed counter summary (line `WHOLE_PROVE_BYTES=`)."""
    path = os.path.join(ROOT, "profiles", "round_data_c3_pmc.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("WHOLE_PROVE_BYTES="):
            return float(line.split("=", 1)[1])
    return None


def cpu_baseline(logD, logN, full_D, full_N):
    """The oracle as it stands, timed on the host cores on a bounded sample of the
    same workload (same generator, smaller D); the figure for the full workload is
    this sample's rate under the fixed work model, and is labelled as such."""
    import numpy as np
    from oracle import pyoracle as orc
    from paper_2404_16109_amd import synth
    cfg = synth.activation_table(rows=1 << (logD - 11), cols=2048, logD=logD, logN=logN)
    T = orc.fr_from_i64(cfg["tx"])
    rho = orc.to_bytes([synth.pair_combiner(cfg["seed"])])[0]
    T = orc.fr_axpy(T, rho, orc.fr_from_i64(cfg["ty"]))
    S = T[cfg["idx"].astype(np.int64)]
    threads = orc.default_threads()
    t0 = time.perf_counter()
    rc, proof, _ = orc.tlookup_prove(cfg["seed"], S, T, threads=threads)
    dt = time.perf_counter() - t0
    assert rc == 0
    out = {"value": fr_mul_model(1 << logD, 1 << logN) / dt, "unit": "Fr-mul/s", "cores": threads, "kind": "oracle",
           "sample": "oracle tlookup_prove timed in this run on the same generator at D=2^%d, N=2^%d: %.1f s wall on %d "
                     "threads; value = that sample's rate under the fixed work model (10 multiplications per element "
                     "and per table row), not a measurement at D=2^%d" % (logD, logN, dt, threads, full_D.bit_length() - 1)}
    rec = recorded_fullsize_oracle()
    if rec:
        out["fullsize_recorded"] = {"seconds": rec["SECONDS"], "cores": int(rec["CORES"]),
                                    "value": fr_mul_model(full_D, full_N) / rec["SECONDS"],
                                    "note": "the oracle's own run at D=2^25, N=2^16 that wrote tests/golden/config3_proof.txt "
                                            "(another machine than this run's: the build container)"}
    return out


def bench_matmul(args, zk, synth, torch, np):
    """Secondary timing: the matmul proof of Section 6.1.1 at the 13B-layer shape."""
    cfg = synth.matmul_operands()
    X, W = cfg["X"], cfg["W"]
    D0, D1 = X.shape
    D2 = W.shape[1]
    vx, vw = zk.Vec(D0 * D1), zk.Vec(D1 * D2)
    assert zk.fr_from_i32(vx, torch.from_numpy(X.astype(np.int32).reshape(-1)).cuda()) == 0
    assert zk.fr_from_i32(vw, torch.from_numpy(W.astype(np.int32).reshape(-1)).cuda()) == 0
    ws = torch.empty(zk.matmul_workspace_bytes(D0, D1, D2), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    first = None
    for _ in range(args.warmup):
        rc, first = zk.matmul_sumcheck_prove(cfg["seed"], vx, D0, D1, vw, D2, ws=ws)
        assert rc == 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        rc, proof = zk.matmul_sumcheck_prove(cfg["seed"], vx, D0, D1, vw, D2, ws=ws)
        assert rc == 0
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    assert first is None or proof == first
    # beside it: the same proof from the 16-bit matrices themselves
    x16 = torch.from_numpy(X.astype(np.int16)).cuda()
    w16 = torch.from_numpy(W.astype(np.int16)).cuda()
    for _ in range(max(args.warmup, 1)):
        rc, proof16 = zk.matmul_sumcheck_prove_i16(cfg["seed"], x16, w16, ws=ws)
        assert rc == 0 and proof16 == proof
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        rc, proof16 = zk.matmul_sumcheck_prove_i16(cfg["seed"], x16, w16, ws=ws)
    torch.cuda.synchronize()
    ms16 = (time.perf_counter() - t0) * 1e3 / args.steps
    muls = D0 * D1 + D1 * D2
    print(json.dumps({
        "metric": "matmul_sumcheck_prove Fr-mul/s at 2048x5120x5120 (secondary timing)",
        "value": muls / (ms * 1e-3), "unit": "Fr-mul/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32x8 (255-bit Montgomery integers)", "data": "synthetic",
        "config": {"workload": "config 4: Y = X W with X 2048x5120, W 5120x5120 (int16 values embedded in Fr)",
                   "fr_mul_model": muls, "bytes_read": 32 * muls, "GBps": 32 * muls / (ms * 1e-3) / 1e9,
                   "from_int16_matrices_ms": ms16}}))


def pair_table_inputs(zk, synth, torch, np, cfg):
    """Inputs into HBM: T = T_X + rho T_Y, S = T[idx] (the looked-up values)."""
    D, N = cfg["D"], cfg["N"]
    T = zk.Vec(N)
    assert zk.fr_from_i32(T, torch.from_numpy(cfg["tx"].astype(np.int32)).cuda()) == 0
    Y = zk.Vec(N)
    assert zk.fr_from_i32(Y, torch.from_numpy(cfg["ty"].astype(np.int32)).cuda()) == 0
    assert zk.fr_axpy(T, T, synth.pair_combiner(cfg["seed"]), Y) == 0
    idx = torch.from_numpy(cfg["idx"].astype(np.int32)).cuda()
    S = zk.Vec(D)
    chunk = 1 << 22
    for s in range(0, D, chunk):
        S.data[:, s:s + chunk] = T.data[:, :N].index_select(1, idx[s:s + chunk].long())
    return S, T, idx


def bench_attention(args, zk, synth, torch, np):
    """Secondary timing: the two digit lookups of the attention workload (2 x 2^28
    lookups, tables of 2^16 pairs) proved with one batched sumcheck, beside the two
    separate proofs."""
    segs = synth.attention_segments()
    D, N = segs[0]["D"], segs[0]["N"]
    Sv, Tv, idx = [], [], []
    for cfg in segs:
        sv, tv, ix = pair_table_inputs(zk, synth, torch, np, cfg)
        Sv.append(sv); Tv.append(tv); idx.append(ix)
    ws = torch.empty(zk.tlookup_batch_workspace_bytes(D, N, 2), dtype=torch.uint8, device="cuda")

    def timed(fn):
        first = None
        for _ in range(args.warmup):
            first = fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            out = fn()
        torch.cuda.synchronize()
        assert first is None or out == first
        return (time.perf_counter() - t0) * 1e3 / args.steps

    def batch():
        rc, proof, _ = zk.tlookup_prove_batch(segs[0]["seed"], Sv, idx, Tv, ws=ws)
        assert rc == 0
        return proof

    def separate():
        out = b""
        for i in range(2):
            rc, proof, _ = zk.tlookup_prove(segs[i]["seed"], Sv[i], idx[i], Tv[i], ws=ws)
            assert rc == 0
            out += proof
        return out

    ms_batch, ms_sep = timed(batch), timed(separate)
    muls = 2 * fr_mul_model(D, N)
    print(json.dumps({
        "metric": "tlookup_prove_batch Fr-mul/s, 2 instances of D=2^28, N=2^16 (secondary timing)",
        "value": muls / (ms_batch * 1e-3), "unit": "Fr-mul/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_batch, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32x8 (255-bit Montgomery integers)", "data": "synthetic",
        "config": {"workload": "config 5: attention scores 40 x 2048 x 2048 padded to 2^28, two 16-bit digit lookups, "
                               "each in its own table of 2^16 pairs, one batched sumcheck",
                   "fr_mul_model": muls, "two_separate_proofs_ms": ms_sep}}))


def link_inputs(zk, synth, torch, np, cfg):
    """The tensors of the closing sumcheck of an attention layer, in HBM: digits
    X^(k), segment outputs Y^(k) = table_k[X^(k)], Y = Y^(0) Y^(1), Z' = -(X^(0) +
    2^16 X^(1)), row sums yhat.  Embedding and products by the library's own
    elementwise calls; only the row sums are added up as integers here."""
    rows, cols = cfg["rows"], cfg["cols"]
    D = rows * cols
    X, Yk = [], []
    ints = {"X": [], "Yk": []}  # the same tensors as integers, for zkattn_link_prove_small
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
    return Zp, X, Y, Yk, yhat, ints


def link_fr_mul_model(D):
    """Multiplications of zkattn_link_prove with two segments, as built: per pair 11
    in the first round (scaling on the fly, two weights, weighted first factor,
    three products), 15 in the second (6 folds more, Z' and the digits no longer
    take part), 13 afterwards; one per entry for each digit tensor's value at the
    final point."""
    return 11 * (D // 2) + 15 * (D // 4) + 13 * (D // 4 - 1) + 2 * D


def bench_link(args, zk, synth, torch, np):
    """Secondary timing: the sumcheck that closes zkAttn-Prove (Protocol 2, last
    step) on the attention workload's tensors."""
    if args.link_rows:
        cfg = synth.attention_link(heads=1, rows=args.link_rows)
    else:
        cfg = synth.attention_link()
    rows, cols = cfg["rows"], cfg["cols"]
    D = rows * cols
    Zp, X, Y, Yk, yhat, ints = link_inputs(zk, synth, torch, np, cfg)
    ws = torch.empty(zk.zkattn_link_workspace_bytes(rows, cols, 2), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()

    def step():
        rc, proof = zk.zkattn_link_prove(cfg["seed"], Zp, X, Y, Yk, yhat, cfg["bases"], rows, cols, ws=ws)
        assert rc == 0, rc
        return proof

    first = None
    for _ in range(args.warmup):
        first = step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        proof = step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    assert first is None or proof == first
    # the proof opens to the tensors it was made from
    rc, _ = zk.zkattn_link_verify(cfg["seed"], proof, rows, cols, cfg["bases"], Zp=Zp, X=X, Y=Y, Yk=Yk, yhat=yhat)
    assert rc == 0, rc
    # the same proof from the tensors as integers
    def small_step():
        rc, got = zk.zkattn_link_prove_small(cfg["seed"], ints["Zp"], ints["X"], ints["Y"], ints["Yk"], yhat, cfg["bases"],
                                             rows, cols, ws=ws)
        assert rc == 0, rc
        return got

    for _ in range(max(args.warmup, 1)):
        assert small_step() == proof
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        small_step()
    torch.cuda.synchronize()
    small_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    muls = link_fr_mul_model(D)
    # all six arrays read once at full size (first round); Y and the two segment outputs then read at size s
    # and written at s/2 for s = D, D/2, ...; the two digit tensors read once more for their final values
    hbm = 32 * (6 * D + 3 * (2 * D + D) + 2 * D)
    print(json.dumps({
        "metric": "zkattn_link_prove Fr-mul/s at %d x %d, 2 segments (secondary timing)" % (rows, cols),
        "value": muls / (ms * 1e-3), "unit": "Fr-mul/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32x8 (255-bit Montgomery integers)", "data": "synthetic",
        "config": {"workload": "config 5: the sumcheck linking Z', two 16-bit digits, their table outputs, the product "
                               "and its row sums, attention scores %d x %d" % (rows, cols),
                   "fr_mul_model": muls, "proof_bytes": len(proof), "from_integer_tensors_ms": small_ms,
                   "algorithmic_hbm_bytes": hbm,
                   "hbm_GBps_algorithmic": hbm / (ms * 1e-3) / 1e9}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--logD", type=int, default=25)
    ap.add_argument("--logN", type=int, default=16)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-logD", type=int, default=21)
    ap.add_argument("--workload", choices=["c3", "c4", "c5", "link"], default="c3",
                    help="c3: tlookup at D=2^25, N=2^16 (the headline metric); c4: matmul sumcheck 2048x5120x5120; "
                         "c5: batched two-segment attention lookup at D=2^28; link: the sumcheck linking the attention "
                         "workload's tensors, 2^17 x 2048 (c4, c5, link: secondary timings)")
    ap.add_argument("--link-rows", type=int, default=0, help="with --workload link: this many rows of 2048 scores "
                    "instead of the full 40 x 2048 (a power of two)")
    ap.add_argument("--no-variants", "--no-by-rows", dest="no_variants", action="store_true",
                    help="skip the timings beside the headline (no hints, exact check, A by gather, integer columns)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (reads 2^30 B, writes 2^30 B) so that rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings can be scaled by a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path needs no second GPU and none is used); "
                 "run with --gpus 1")

    import numpy as np
    import torch
    import paper_2404_16109_amd as zk
    from paper_2404_16109_amd import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    if args.workload == "c4":
        return bench_matmul(args, zk, synth, torch, np)
    if args.workload == "c5":
        return bench_attention(args, zk, synth, torch, np)
    if args.workload == "link":
        return bench_link(args, zk, synth, torch, np)
    D, N = 1 << args.logD, 1 << args.logN
    rows = 2048 if args.logD >= 25 else max(1, (D * 11) // (16 * 2048))
    cols = 11008 if args.logD >= 25 else 2048
    cfg = synth.activation_table(rows=rows, cols=cols, logD=args.logD, logN=args.logN)

    S, T, idx = pair_table_inputs(zk, synth, torch, np, cfg)
    ws = torch.empty(zk.tlookup_workspace_bytes(D, N), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()

    def step():
        rc, proof, info = zk.tlookup_prove(cfg["seed"], S, idx, T, ws=ws)
        assert rc == 0, rc
        return proof, info

    if args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def timed(fn, steps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            out = fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, out

    # -- the headline: W warm-up steps, then exactly K timed steps, nothing else going on
    first = None
    for _ in range(args.warmup):
        first, _ = step()
    ms, (proof, info) = timed(step, args.steps)
    assert first is None or proof == first            # exact arithmetic: every run gives the same bytes
    assert info["sum_A"] == info["sum_mB"]            # log-derivative identity at beta

    # -- beside it (each checked to give the same proof, two warm-up calls, then timed)
    beside = {}
    if not args.no_variants:
        X = torch.from_numpy(cfg["tx"].astype(np.int32)).cuda()[idx.long()].contiguous()
        Y = torch.from_numpy(cfg["ty"].astype(np.int32)).cuda()[idx.long()].contiguous()
        rho = synth.pair_combiner(cfg["seed"])
        ws_small = torch.empty(zk.tlookup_small_workspace_bytes(D, N), dtype=torch.uint8, device="cuda")
        variants = {
            # rows found through the hash of T, every S_i compared with its row while counting
            "unhinted_ms_per_step": lambda: zk.tlookup_prove(cfg["seed"], S, None, T, ws=ws)[:2],
            # hints given, but every S_i compared with T[idx_i] up front instead of through the identity
            "checked_ms_per_step": lambda: zk.tlookup_prove_checked(cfg["seed"], S, idx, T, ws=ws)[:2],
            # A read off the table-side inverses instead of inverting D elements
            "by_rows_ms_per_step": lambda: zk.tlookup_prove_by_rows(cfg["seed"], S, idx, T, ws=ws)[:2],
            # the tensor as two int32 columns (8 bytes per entry instead of 32)
            "small_ms_per_step": lambda: zk.tlookup_prove_small(cfg["seed"], X, Y, rho, idx, T, ws=ws_small)[:2],
        }
        for name, fn in variants.items():
            for _ in range(2):
                rc, got = fn()
                assert rc == 0 and got == proof, name
            beside[name], _ = timed(fn, args.steps)

        # Two proofs in flight: two host threads, each with a stream and a workspace of its own, proving the same
        # inputs.  One proof alone leaves the device idle while the host answers a round (latency_share below) and
        # keeps either the ALU or HBM waiting in most kernels; a second proof fills those holes.  Reported per proof.
        import threading
        ws2 = torch.empty(zk.tlookup_workspace_bytes(D, N), dtype=torch.uint8, device="cuda")
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        failures = []

        def worker(which, steps):
            try:
                with torch.cuda.stream(streams[which]):
                    for _ in range(steps):
                        rc, got, _ = zk.tlookup_prove(cfg["seed"], S, idx, T, ws=(ws, ws2)[which])
                        if rc != 0 or got != proof:
                            failures.append((which, rc))
            except Exception as e:  # a thread must not die silently
                failures.append((which, repr(e)))

        def both(steps):
            threads = [threading.Thread(target=worker, args=(w, steps)) for w in range(2)]
            for t in threads:
                t.start()
            for t in threads:
                t.join()

        both(2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        both(args.steps)
        torch.cuda.synchronize()
        beside["two_in_flight_ms_per_proof"] = (time.perf_counter() - t0) * 1e3 / (2 * args.steps)
        assert not failures, failures
        del ws2

    # -- where the time goes: a separate pass with the library's own event pairs on the launch stream
    zk.zkmi_profile_reset()
    zk.zkmi_profile_enable(True)
    psteps = max(1, min(args.steps, 5))
    timed(step, psteps)
    zk.zkmi_profile_enable(False)
    names = ("total", "count", "inverse", "digest", "round_data", "round_table", "round_data29", "round_small")
    phases = {}
    for name in names:
        rc, recs, total_ms = zk.zkmi_profile_query(name)
        phases[name] = {"records": recs, "ms_per_step": total_ms / psteps}

    # the dominant kernel: k_round_data29, one launch per large folding round
    rd = phases["round_data29"]
    launches = rd["records"] / psteps
    avg_launch_s = rd["ms_per_step"] * 1e-3 / max(launches, 1)
    pairs29, muls29, moved29 = round29_work(D, N)
    mads_per_launch = muls29 * MADS_PER_FR_MUL / max(launches, 1)
    bytes_per_launch = moved29 / max(launches, 1)
    alu = mads_per_launch / avg_launch_s if avg_launch_s > 0 else 0.0
    hbm = bytes_per_launch / avg_launch_s if avg_launch_s > 0 else 0.0
    traffic = measured_traffic()
    # the whole prove against both roofs, by the fixed models: 112 multiply-adds per model multiplication, and the
    # bytes that must move even with perfect fusion (292 per element of S: hints, the inversion's three passes, every
    # round's arrays read once and written at half size)
    whole_mads = fr_mul_model(D, N) * MADS_PER_FR_MUL
    whole_bytes = WHOLE_PROVE_BYTES_PER_ELEMENT * D
    kernels_ms = sum(phases[k]["ms_per_step"] for k in names if k != "total")
    total_ms = phases["total"]["ms_per_step"]
    whole = {
        "alu_frac": whole_mads / (ms * 1e-3) / PEAK_MAD_PER_S,
        "hbm_frac": whole_bytes / (ms * 1e-3) / PEAK_HBM_BYTES_PER_S,
        "fr_mul_per_s": fr_mul_model(D, N) / (ms * 1e-3),
        "hbm_GBps_algorithmic": whole_bytes / (ms * 1e-3) / 1e9,
        "hbm_bytes_measured": measured_whole_prove_traffic(),
        # the share of a prove in which neither roof is touched: the device idle between dependent launches (waiting
        # for the transcript on the host) plus the kernels of the rounds that are bound by latency
        "latency_share": (max(total_ms - kernels_ms, 0.0) + phases["round_small"]["ms_per_step"]) / total_ms if total_ms else None,
    }
    if whole["hbm_bytes_measured"]:
        whole["hbm_frac_measured"] = whole["hbm_bytes_measured"] / (ms * 1e-3) / PEAK_HBM_BYTES_PER_S
    # every phase of the prove against the HBM roof, by the bytes it cannot avoid (per element of S: the hints read
    # once; S read and A written by the inversion, its prefix products written and read once; A read by the hash tree;
    # A and S read by the pass that serves the first two rounds; the folding rounds by round29_work)
    phase_bytes = {"count": 4 * D, "inverse": 96 * D, "digest": 32 * D, "round_data": 64 * D, "round_data29": moved29}
    phase_bound = {"count": "LDS atomics", "inverse": "hbm", "digest": "alu (SHA-256 instruction issue)",
                   "round_data": "alu (two wavefronts per SIMD)", "round_data29": "hbm and alu, balanced"}
    whole["phases"] = {
        k: {"ms": round(phases[k]["ms_per_step"], 4), "algorithmic_bytes": b, "bound": phase_bound[k],
            "hbm_frac": (b / (phases[k]["ms_per_step"] * 1e-3) / PEAK_HBM_BYTES_PER_S) if phases[k]["ms_per_step"] > 0 else None}
        for k, b in phase_bytes.items()}
    out = {
        "metric": "tlookup_prove Fr-mul/s at D=2^%d, N=2^%d (wall ms in ms_per_step)" % (args.logD, args.logN),
        "value": fr_mul_model(D, N) / (ms * 1e-3),
        "unit": "Fr-mul/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32x8 (255-bit Montgomery integers)", "data": "synthetic",
        "config": {"workload": "config 3: tlookup SwiGLU/activation pair table at 7B-FFN shape, "
                               "%d x %d activations padded to D=2^%d, N=2^%d" % (rows, cols, args.logD, args.logN),
                   "path": "tlookup_prove with row hints (idx given: counts from the hints, S checked against them through "
                           "sum A = sum m B after the first round); the variants beside it prove the same bytes",
                   "D": D, "N": N, "proof_bytes": len(proof), "fr_mul_model": fr_mul_model(D, N)},
        "phases_ms": {k: round(v["ms_per_step"], 4) for k, v in phases.items()},
        "commitment_standin_ms": round(phases["digest"]["ms_per_step"], 4),
        "roofline": {"bound": "hbm" if hbm / PEAK_HBM_BYTES_PER_S >= alu / PEAK_MAD_PER_S else "alu",
                     "kernel": "k_round_data29 (the large folding rounds, %d launches per prove)" % len(rounds_on_29_bits(D, N)),
                     "achieved": hbm / 1e9, "peak": PEAK_HBM_BYTES_PER_S / 1e9, "unit": "GB/s",
                     "frac": hbm / PEAK_HBM_BYTES_PER_S, "traffic": traffic,
                     "launches_per_step": launches, "avg_launch_ms": avg_launch_s * 1e3,
                     "algorithmic_bytes_per_launch": bytes_per_launch,
                     "alu": {"achieved": alu / 1e12, "peak": PEAK_MAD_PER_S / 1e12, "unit": "T int32-mad/s",
                             "frac": alu / PEAK_MAD_PER_S, "fr_mul_per_pair_model": 9, "fr_mul_per_pair_executed": 8},
                     "whole_prove": whole},
    }
    out.update(beside)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.cpu_logD, min(args.logN, args.cpu_logD), D, N)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
