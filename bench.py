#!/usr/bin/env python3
"""Benchmark of the tlookup prover hot path on one MI355X.

A "step" is one whole `tlookup_prove` call (multiplicities, digest of m, both
batch inversions, eq tables, all sumcheck rounds with folding, transcript) on
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


def fr_mul_model(D, N):
    return 10 * D + 10 * N


def rounds_on_29_bits(D, N):
    """The rounds the dominant kernel (k_round_data29) runs: after the first, before
    the table's variables, while more than 256 pairs remain."""
    n, h = D.bit_length() - 1, (D // N).bit_length() - 1
    return [k for k in range(1, h) if (D >> (k + 1)) > 256]


def round29_pairs(D, N):
    return sum(D >> (k + 1) for k in rounds_on_29_bits(D, N))


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


def cpu_baseline(logD, logN):
    """The oracle as it stands, timed on the host cores on a bounded sample of the
    same workload (same generator, smaller D)."""
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
    return {"value": fr_mul_model(1 << logD, 1 << logN) / dt, "unit": "Fr-mul/s", "cores": threads, "kind": "oracle",
            "sample": "oracle tlookup_prove on the same generator at D=2^%d, N=2^%d: %.1f s wall" % (logD, logN, dt)}


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
    ap.add_argument("--cpu-logD", type=int, default=19)
    ap.add_argument("--workload", choices=["c3", "c4", "c5", "link"], default="c3",
                    help="c3: tlookup at D=2^25, N=2^16 (the headline metric); c4: matmul sumcheck 2048x5120x5120; "
                         "c5: batched two-segment attention lookup at D=2^28; link: the sumcheck linking the attention "
                         "workload's tensors, 2^17 x 2048 (c4, c5, link: secondary timings)")
    ap.add_argument("--link-rows", type=int, default=0, help="with --workload link: this many rows of 2048 scores "
                    "instead of the full 40 x 2048 (a power of two)")
    ap.add_argument("--no-by-rows", action="store_true", help="skip the tlookup_prove_by_rows timing beside the headline")
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

    first = None
    for _ in range(args.warmup):
        first, _ = step()
    zk.zkmi_profile_reset()
    zk.zkmi_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        proof, info = step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    zk.zkmi_profile_enable(False)
    assert first is None or proof == first            # exact arithmetic: every run gives the same bytes
    assert info["sum_A"] == info["sum_mB"]            # log-derivative identity at beta

    ms = dt * 1e3 / args.steps
    # beside the headline: the same proof with A read off the table-side inverses
    ms_rows = None
    if not args.no_by_rows:
        for _ in range(2):
            rc, proof_rows, _ = zk.tlookup_prove_by_rows(cfg["seed"], S, idx, T, ws=ws)
            assert rc == 0 and proof_rows == proof
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            rc, proof_rows, _ = zk.tlookup_prove_by_rows(cfg["seed"], S, idx, T, ws=ws)
        torch.cuda.synchronize()
        ms_rows = (time.perf_counter() - t0) * 1e3 / args.steps
    phases = {}
    for name in ("total", "count", "inverse", "round_data", "round_table", "round_data29"):
        rc, recs, total_ms = zk.zkmi_profile_query(name)
        phases[name] = {"records": recs, "ms_per_step": total_ms / args.steps}
    # round_data: every round kernel with a data side, the dominant one (round_data29) included
    phases["round_data"] = {"records": phases["round_data"]["records"] + phases["round_data29"]["records"],
                            "ms_per_step": phases["round_data"]["ms_per_step"] + phases["round_data29"]["ms_per_step"]}
    # the dominant kernel: k_round_data29, one launch per large folding round
    rd = phases["round_data29"]
    launches = rd["records"] / args.steps
    avg_launch_s = rd["ms_per_step"] * 1e-3 / max(launches, 1)
    pairs29 = round29_pairs(D, N)
    mads_per_launch = pairs29 * (ROUND_DATA_FR_MUL_PER_PAIR_EVAL + ROUND_DATA_FR_MUL_PER_PAIR_FOLD) * MADS_PER_FR_MUL / max(launches, 1)
    bytes_per_launch = pairs29 * 12 * 32 / max(launches, 1)  # per pair: four entries of A and of S read, two of each written
    achieved = mads_per_launch / avg_launch_s if avg_launch_s > 0 else 0.0
    out = {
        "metric": "tlookup_prove Fr-mul/s at D=2^%d, N=2^%d (wall ms in ms_per_step)" % (args.logD, args.logN),
        "value": fr_mul_model(D, N) / (ms * 1e-3),
        "unit": "Fr-mul/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32x8 (255-bit Montgomery integers)", "data": "synthetic",
        "config": {"workload": "config 3: tlookup SwiGLU/activation pair table at 7B-FFN shape, "
                               "%d x %d activations padded to D=2^%d, N=2^%d" % (rows, cols, args.logD, args.logN),
                   "D": D, "N": N, "proof_bytes": len(proof), "fr_mul_model": fr_mul_model(D, N)},
        "phases_ms": {k: round(v["ms_per_step"], 4) for k, v in phases.items()},
        "by_rows_ms_per_step": ms_rows,
        "roofline": {"bound": "alu", "kernel": "k_round_data29 (the large folding rounds, %d launches per prove)" % len(rounds_on_29_bits(D, N)),
                     "achieved": achieved / 1e12, "peak": PEAK_MAD_PER_S / 1e12, "unit": "T int32-mad/s",
                     "frac": achieved / PEAK_MAD_PER_S, "traffic": measured_traffic(),
                     "launches_per_step": launches, "avg_launch_ms": avg_launch_s * 1e3,
                     "algorithmic_bytes_per_launch": bytes_per_launch,
                     "hbm_GBps_algorithmic": bytes_per_launch / avg_launch_s / 1e9 if avg_launch_s > 0 else 0.0},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.cpu_logD, min(args.logN, args.cpu_logD))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
