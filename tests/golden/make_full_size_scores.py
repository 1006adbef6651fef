#!/usr/bin/env python3
"""Writes tests/golden/full_size_scores.npz: float64 oracle scores of whole users of the
full-size workloads (C3: every user; C4, C5 and the X variants: the users listed below).

Imports only `oracle` and `synth`: every stored value is the CPU oracle's full recompute
(full inference over [prefix | suffix | candidates], no cache) on the seeded inputs of batch 0 of the
workload.  The GPU tests compare the HIP path's scores with these element by element, so that the
box that holds the GPU does not spend minutes of float64 CPU time per run.

    python tests/golden/make_full_size_scores.py [--only C5] [--threads 8]

Entries already present in the file are kept and skipped (delete the file to regenerate all).
Takes about half an hour on 8 cores; the longest users (16 384 prefix tokens) need about 15 GiB.
"""
from __future__ import annotations

import argparse
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

OUT = os.path.join(HERE, "full_size_scores.npz")

# workload -> users whose scores are stored.  C5 (batch 0): both users at the 16 384-token clip (41 cached, 61
# uncached), the next-longest (16), the shortest cached (32) and uncached (48) users, uncached users of middle
# length with many candidates (9) and a long suffix (51), a cached user with the longest suffix (3), and a short
# cached user with many candidates (4).
USERS = {
    "C3": list(range(16)),
    "C4": [0, 5, 9, 13, 18, 22, 27, 31],
    "C5": [61, 41, 16, 32, 48, 9, 51, 3, 4],
    "X1": [3],
    "X2": [7],
    "X3": [9],
    "X4": [4],
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--only", action="append", default=None, help="workload(s) to (re)compute")
    ap.add_argument("--threads", type=int, default=None)
    args = ap.parse_args()

    import torch

    import oracle
    import synth
    from synth.generator import user_slices

    if args.threads:
        torch.set_num_threads(args.threads)
    store = {}
    if os.path.exists(OUT):
        with np.load(OUT, allow_pickle=False) as z:
            store = {k: z[k] for k in z.files}
    for name in (args.only or list(USERS)):
        wl = synth.WORKLOADS[name]
        cfg = wl.model
        todo = [u for u in USERS[name] if f"{name}/u{u}" not in store]
        if not todo:
            continue
        weights = synth.make_weights(cfg, wl.seed)
        batch = synth.make_batch(wl, 0)
        for u in todo:
            p, s, c = user_slices(batch, u)
            t0 = time.time()
            ref = oracle.full_recompute(cfg, weights, p, s, c)
            store[f"{name}/u{u}"] = np.asarray(ref, dtype=np.float64)
            store[f"{name}/u{u}/shape"] = np.asarray([len(p), len(s), len(c)], dtype=np.int64)
            print(f"{name} user {u}: prefix {len(p)}, suffix {len(s)}, candidates {len(c)}: {time.time() - t0:.1f}s", flush=True)
            np.savez(OUT, **store)     # after every user, so that an interrupted run keeps its work
    return 0


if __name__ == "__main__":
    sys.exit(main())
