"""Writes tests/golden/cfg3_batch1_x0.txt: the final latent x_0 of workload configuration 3
(DiT-XL/2-shaped, 28 blocks, guidance 4, 50-step DDIM, conservative n = 4) for batch 1, computed by the
CPU oracle alone (fp64, Algorithm 2 of the paper step by step).  Nothing from the HIP library is
imported or called.  Takes about half an hour on 8 cores.

    python tests/golden/make_cfg3_sample.py
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle.ref import Oracle                      # noqa: E402
from paper_2603_25872_amd import inputs as I       # noqa: E402  (seeded input generators only)


def main():
    cfg = I.config(3)
    dit, sd = cfg["dit"], cfg["sched"]
    orc = Oracle(64)
    w = I.weights(dit, 3)
    xT = I.latent_noise(dit, 1, 3)
    cond = I.conditioning(dit, 1, 3)
    null = I.conditioning(dit, 1, 3, null=True)
    t0 = time.perf_counter()
    x0 = orc.sample_dit(dit, w, sd, cfg["mode"], cfg["n"], xT, cond, null, cfg["guidance"])
    dt = time.perf_counter() - t0
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg3_batch1_x0.txt")
    header = ("x_0 of configuration 3, batch 1 (seeded inputs of stream 3), CPU oracle fp64, %d threads, %.0f s; "
              "shape %s, C order" % (orc.threads(), dt, tuple(x0.shape)))
    np.savetxt(out, np.asarray(x0, np.float64).ravel(), fmt="%.10e", header=header)
    print("wrote", out, "in %.0f s" % dt)


if __name__ == "__main__":
    main()
