"""Writes tests/golden/cfg2_x0.txt: the final latents x_0 of workload configuration 2 exactly as
specified (DiT-S-shaped, 12 blocks, hidden 384, 6 heads, latent 4x32x32, 50-step DDIM, aggressive
n = 3, batch 4, no guidance), computed by the CPU oracle alone (fp64, Algorithm 1 of the paper step
by step).  Nothing from the HIP library is imported or called.  About 3 minutes on 8 cores.

    python tests/golden/make_cfg2_sample.py
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
    cfg = I.config(2)
    dit, sd, B = cfg["dit"], cfg["sched"], cfg["batch"]
    orc = Oracle(64)
    w = I.weights(dit, 2)
    xT = I.latent_noise(dit, B, 2)
    cond = I.conditioning(dit, B, 2)
    t0 = time.perf_counter()
    x0 = orc.sample_dit(dit, w, sd, cfg["mode"], cfg["n"], xT, cond)
    dt = time.perf_counter() - t0
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg2_x0.txt")
    header = ("x_0 of configuration 2, batch %d (seeded inputs of stream 2), CPU oracle fp64, %d threads, %.0f s; "
              "shape %s, C order" % (B, orc.threads(), dt, tuple(x0.shape)))
    np.savetxt(out, np.asarray(x0, np.float64).ravel(), fmt="%.8e", header=header)
    print("wrote", out, "in %.0f s" % dt)


if __name__ == "__main__":
    main()
