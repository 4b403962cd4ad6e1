#!/usr/bin/env python3
"""Writes the stored expectations for the full-size gradient-descent runs.

Calls only the seeded generators and the CPU oracle (never the device library).  The oracle needs
minutes for these sizes, which is why its results are stored instead of recomputed in every test
run.  Each file records a checksum of the labels so that a test can prove it feeds the device the
same problem.

    python tests/golden/make_golden.py [config2] [config3] [config4]

Outputs (float64): <name>_gd.npz with W (c_T x m), losses (iters x m), y_sha256, and for config3
also the Gram matrix T^T T.
"""
import hashlib
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import datagen  # noqa: E402
import oracle  # noqa: E402


def sha(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def run(name: str) -> None:
    t0 = time.time()
    sch = getattr(datagen, name)()
    tg = oracle.Target(sch)
    kind = "logistic" if name == "config2" else "linear"
    y = datagen.finish_labels(kind, oracle.lmm(tg, sch.extras["w_star"].reshape(-1, 1)), sch.extras["noise"])
    lr = sch.extras["lr"]
    iters = int(sch.extras["iters"][0])
    print(f"{name}: table {tg.T32.shape} ready after {time.time() - t0:.0f} s; {iters} iterations x {len(lr)} models", flush=True)
    W, losses = oracle.gd(tg, kind, y, np.zeros((sch.c_T, len(lr))), lr, iters)
    out = {"W": W, "losses": losses, "y_sha256": np.array(sha(y)), "lr": lr}
    if name == "config3":
        out["gram"] = oracle.crossprod(tg)
    np.savez_compressed(os.path.join(HERE, f"{name}_gd.npz"), **out)
    print(f"{name}: done in {time.time() - t0:.0f} s", flush=True)


if __name__ == "__main__":
    for n in (sys.argv[1:] or ["config3", "config4", "config2"]):
        run(n)
