#!/usr/bin/env python3
"""Writes tests/golden/fullsize_<workload>.npz: the ORACLE's target-independent row statistics
(row max, logsumexp, top-2 gap, argmax) of the full-size synthetic workloads, so that the GPU
parity tests at full size can compare every row without redoing the fp64 vocabulary sweep.

Calls only oracle/ and the seeded input generators; nothing here comes from the HIP path.

    python tests/golden/make_fullsize_stats.py [workload ...]

Rows whose two largest logits nearly tie (gap < tests.helpers.GAP_GUARD) are re-drawn, each
from its own seeded stream, until none is left; `row_attempts` records how often, and
synth.make_head(..., row_attempts=...) rebuilds exactly the same inputs.
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import cat_oracle as O                      # noqa: E402
from paper_2605_08632_amd import synth                  # noqa: E402
from tests.helpers import GAP_GUARD                     # noqa: E402

FULLSIZE = ("c2_llama1b_bf16", "c3_qwen06b_bf16", "c4_8bwidth_bf16")


def main(names):
    for name in names:
        wl = synth.WORKLOADS[name]
        t0 = time.time()
        attempts = np.zeros(wl.T, dtype=np.int64)
        head = synth.make_head(wl.seed, wl.T, wl.d, wl.V, wl.dtype)
        W64 = head.W.astype(np.float64)
        zeros = np.zeros(wl.T, dtype=np.int64)
        st = O.head_stats(head.H, None, zeros, W64=W64)
        rounds = 0
        while True:
            near = np.nonzero(st["gap"] < GAP_GUARD)[0]
            if len(near) == 0:
                break
            rounds += 1
            attempts[near] += 1
            head = synth.make_head(wl.seed, wl.T, wl.d, wl.V, wl.dtype, row_attempts=attempts)
            sub = O.head_stats(head.H[near], None, zeros[:len(near)], W64=W64)
            for k in ("m", "lse", "gap", "argmax"):
                st[k][near] = sub[k]
        out = os.path.join(ROOT, "tests", "golden", f"fullsize_{name}.npz")
        np.savez_compressed(out, m=st["m"], lse=st["lse"], gap=st["gap"],
                            argmax=st["argmax"].astype(np.int32), row_attempts=attempts.astype(np.int8),
                            gap_guard=np.float64(GAP_GUARD))
        print(f"{name}: {int((attempts > 0).sum())} rows re-drawn in {rounds} rounds, "
              f"{time.time() - t0:.0f} s -> {out} ({os.path.getsize(out) / 1024:.0f} KiB)", flush=True)


if __name__ == "__main__":
    main(sys.argv[1:] or FULLSIZE)
