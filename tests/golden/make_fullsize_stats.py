#!/usr/bin/env python3
"""Writes tests/golden/fullsize_<workload>.npz: the ORACLE's target-independent row statistics
(row max, logsumexp, top-2 gap, argmax) of the full-size synthetic workloads, so that the GPU
parity tests at full size can compare every row without redoing the fp64 vocabulary sweep.

Calls only oracle/ and the seeded input generators; nothing here comes from the HIP path.

    python tests/golden/make_fullsize_stats.py [workload ...]
    python tests/golden/make_fullsize_stats.py kd:<workload>:<teacher width>

The second form writes fullsize_kd_<workload>_dt<width>.npz: the teacher head's logsumexp and
KL(teacher || draft) of every row (both target-independent) for the two-head loss, from the
workload's stored draft inputs plus synth.make_teacher; the draft statistics file must exist.

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


def main_kd(name, dt):
    from oracle import cat_kd_oracle as KD
    wl = synth.WORKLOADS[name]
    t0 = time.time()
    base = np.load(os.path.join(ROOT, "tests", "golden", f"fullsize_{name}.npz"))
    head = synth.make_head(wl.seed, wl.T, wl.d, wl.V, wl.dtype, row_attempts=np.asarray(base["row_attempts"]))
    teacher = synth.make_teacher(wl.seed, head, dt)
    st = KD.kd_stats(head.H, head.W.astype(np.float64), teacher.H, teacher.W.astype(np.float64),
                     np.zeros(wl.T, dtype=np.int64))
    assert np.allclose(st["lse"], base["lse"], rtol=0, atol=1e-9)      # same draft inputs as the stored file
    out = os.path.join(ROOT, "tests", "golden", f"fullsize_kd_{name}_dt{dt}.npz")
    np.savez_compressed(out, lse_t=st["lse_t"], kd=st["kd"], teacher_d=np.int64(dt))
    print(f"kd {name} dt={dt}: {time.time() - t0:.0f} s -> {out} ({os.path.getsize(out) / 1024:.0f} KiB)", flush=True)


if __name__ == "__main__":
    args = sys.argv[1:]
    for a in [a for a in args if a.startswith("kd:")]:
        _, name, dt = a.split(":")
        main_kd(name, int(dt))
    plain = [a for a in args if not a.startswith("kd:")]
    if plain or not args:
        main(plain or FULLSIZE)
