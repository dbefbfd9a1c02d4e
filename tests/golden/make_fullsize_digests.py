#!/usr/bin/env python3
"""Writes the expected tlookup proofs of the full-size workloads (config 3:
D = 2^25, and the two segments of config 5: D = 2^28) by running the CPU oracle.

Calls only `oracle/` and the seeded input generators; nothing here touches the
device library.  Takes about two minutes for config 3 and tens of minutes (and
about 35 GiB of RAM) per config-5 segment on 8 cores.

    python tests/golden/make_fullsize_digests.py c3
    python tests/golden/make_fullsize_digests.py c5
"""
import hashlib
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import pyoracle as orc            # noqa: E402
from paper_2404_16109_amd import synth        # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def run(cfg, out_name):
    t0 = time.time()
    T = orc.fr_from_i64(cfg["tx"])
    rho = orc.to_bytes([synth.pair_combiner(cfg["seed"])])[0]
    T = orc.fr_axpy(T, rho, orc.fr_from_i64(cfg["ty"]))
    S = T[cfg["idx"].astype(np.int64)]
    rc, proof, info = orc.tlookup_prove(cfg["seed"], S, T, threads=os.cpu_count())
    assert rc == 0, rc
    with open(os.path.join(HERE, out_name), "w") as f:
        f.write("# tlookup proof of workload %s (D=%d, N=%d) written by the CPU oracle\n" % (cfg["name"], cfg["D"], cfg["N"]))
        f.write("# through tests/golden/make_fullsize_digests.py; first line the SHA-256 of the proof, second the proof.\n")
        f.write(hashlib.sha256(proof).hexdigest() + "\n")
        f.write(proof.hex() + "\n")
    print("%s: %d bytes, %.0f s" % (out_name, len(proof), time.time() - t0), flush=True)


if __name__ == "__main__":
    which = sys.argv[1] if len(sys.argv) > 1 else "c3"
    if which == "c3":
        run(synth.activation_table(), "config3_proof.txt")
    elif which == "c5":
        for k, cfg in enumerate(synth.attention_segments()):
            run(cfg, "config5_seg%d_proof.txt" % k)
    else:
        sys.exit("usage: make_fullsize_digests.py c3|c5")
