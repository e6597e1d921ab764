"""Writes tests/golden/cfg2_samplers_x0.txt: final latents of workload configuration 2 at its stated shape
(DiT-S-shaped, 12 blocks, 32x32 latent, 50 steps, aggressive n = 3, batch 4) under the three other samplers of
the section "Skip Transitions": stochastic DDIM with eta = 0.5 (Eq. ddim_skip_reverse with variance), the
DDPM Bayes-posterior skip (Eq. ddpm_skip_reverse), both with the fresh noise of the counter-based stream
(seed 4242, fields from 0; the oracle draws it with its own generator), and the Euler skip with time shift 3.
Computed by the CPU oracle alone (fp64); nothing from the HIP library is imported or called.  Samples 0 and 3
of the batch are stored.  About 4 minutes per sampler on 8 cores.

    python tests/golden/make_cfg2_samplers.py
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle.ref import Oracle                      # noqa: E402
from paper_2603_25872_amd import inputs as I       # noqa: E402  (seeded input generators only)

SEED, KEEP = 4242, (0, 3)
SAMPLERS = [("ddim_eta0.5", dict(eta=0.5)), ("ddpm", dict(sampler=1)), ("euler_shift3", dict(sampler=2, shift=3.0))]


def main():
    cfg = I.config(2)
    dit, B = cfg["dit"], cfg["batch"]
    orc = Oracle(64)
    w = orc.prepare_weights(I.weights(dit, 2))
    xT = I.latent_noise(dit, B, 2)
    cond = I.conditioning(dit, B, 2)
    lines = []
    for name, extra in SAMPLERS:
        sd = dict(cfg["sched"], **extra)
        cnt = orc.noise_count(sd, cfg["mode"], cfg["n"])
        z = orc.normal_fill(SEED, 0, cnt, xT.size).reshape((cnt,) + xT.shape) if cnt and extra.get("sampler") != 2 else None
        t0 = time.perf_counter()
        x0 = orc.sample_dit(dit, w, sd, cfg["mode"], cfg["n"], xT, cond, z=z)
        print("%s done in %.0f s" % (name, time.perf_counter() - t0), flush=True)
        for b in KEEP:
            lines.append("# %s sample %d" % (name, b))
            lines += ["%.8e" % float(v) for v in np.asarray(x0[b], np.float64).ravel()]
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg2_samplers_x0.txt")
    with open(out, "w") as f:
        f.write("# x_0 of configuration 2 (batch %d, seeded inputs of stream 2) under three samplers, CPU oracle fp64, %d threads;\n"
                "# noise stream seed %d, field 0 onwards; per record the %d values of one sample, C order\n"
                % (B, orc.threads(), SEED, x0[0].size))
        f.write("\n".join(lines) + "\n")
    print("wrote", out)


if __name__ == "__main__":
    main()
