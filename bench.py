"""Throughput of the DRiffusion hot path on one MI355X.

One "step" is one drf_sample call: the whole draft-and-refine loop (all S sampling
steps: batched DiT passes + fused guidance/refine/draft updates) over one batch of
synthetic latents, inputs resident in HBM.  Default workload: configuration 3
(DiT-XL/2-shaped, bf16, guidance 4, 50-step DDIM, conservative n=4, batch 8).

Prints ONE JSON line: eps-evals/s over the whole call, ms per step, the roofline of the
dominant kernel family (bf16 MFMA GEMM) measured with HIP events on the library's
stream during one extra instrumented call, and the CPU oracle timed on a bounded
sample of the same workload (one slot evaluation of the same DiT)."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# Bytes the bf16 GEMM launches of one configuration-3 call move past the L2, per launch on average: rocprofv3 FETCH_SIZE
# and WRITE_SIZE, each scaled by what the same counter reads for a plain 1 GiB copy
# (profiles/drf_sample_cfg3_pmc_traffic_mfma.txt).  Only valid for the default workload.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = {3: 1.873e8}


def slot_eval_flops(dit):
    """Algorithmic flops of one slot evaluation (2 M N K, unpadded head dim)."""
    D, L, R = dit["hidden"], dit["depth"], dit["mlp_ratio"]
    T = (dit["lat_h"] // dit["patch"]) * (dit["lat_w"] // dit["patch"])
    P = dit["in_ch"] * dit["patch"] ** 2
    per = 2 * T * D * (3 * D) + 2 * T * D * D + 2 * 2 * T * D * R * D + 4 * T * T * D
    if dit["cond"] == 2:
        per += 2 * 2 * T * D * D + 4 * T * dit["ctx_len"] * D
    return L * per + 2 * 2 * T * D * P


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=3, help="workload configuration 1..5")
    ap.add_argument("--n", type=int, default=None, help="override the block size n")
    ap.add_argument("--mode", type=int, default=None, help="0 conservative, 1 aggressive")
    ap.add_argument("--batch", type=int, default=None, help="override the batch size")
    ap.add_argument("--sampler", type=int, default=0, help="0 DDIM, 1 DDPM posterior, 2 Euler (velocity net)")
    ap.add_argument("--eta", type=float, default=0.0, help="DDIM: variance scale of the skip transitions")
    ap.add_argument("--shift", type=float, default=1.0, help="Euler: time shift of the sigma grid")
    ap.add_argument("--seed", type=int, default=1, help="seed of the library's noise stream (stochastic samplers)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run three plain 1 GiB device-to-device copies: the kernel of known size against "
                         "which the FETCH_SIZE / WRITE_SIZE counters of a profiler run are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; the paper's n devices are n batch-slot groups of a "
                 "single pass, so --gpus must be 1")

    import numpy as np
    import torch
    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_copy": 1 << 30, "bytes_written_per_copy": 1 << 30, "copies": 3}}))
        return
    from paper_2603_25872_amd import build as lib_build, drf, inputs as I
    lib_build.ensure_built()                       # loads what is built; compiles only if nothing is

    cfg = I.config(args.config)
    dit, sd = cfg["dit"], dict(cfg["sched"], sampler=args.sampler, eta=args.eta, shift=args.shift)
    n = cfg["n"] if args.n is None else args.n
    mode = cfg["mode"] if args.mode is None else args.mode
    B, S = (cfg["batch"] if args.batch is None else args.batch), sd["steps"]
    stochastic = args.sampler == 1 or (args.sampler == 0 and args.eta != 0.0)
    default_workload = (args.n is None and args.mode is None and args.batch is None and args.sampler == 0
                        and args.eta == 0.0)
    g = 2 if cfg["guidance"] else 1
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    w = I.weights(dit, args.config)
    den = drf.Denoiser(dit, w)
    den.reserve(n * g * B)
    xT = torch.from_numpy(I.latent_noise(dit, B, args.config)).cuda()
    cond = torch.from_numpy(I.conditioning(dit, B, args.config)).cuda()
    null = torch.from_numpy(I.conditioning(dit, B, args.config, null=True)).cuda() if cfg["guidance"] else None
    out = torch.empty_like(xT)

    def step():
        if stochastic:      # fresh noise generated inside the update kernel from the library's stream
            den.sample_noise(sd, mode, n, xT, cond, null, cfg["guidance"] or 0.0, seed=args.seed, out=out)
        else:
            den.sample(sd, mode, n, xT, cond, null, cfg["guidance"] or 0.0, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert bool(torch.isfinite(out).all())

    evals = S * B * g                                   # slot evaluations per call
    ms_step = dt / args.steps * 1e3
    flops_call = evals * slot_eval_flops(dit)
    result = {
        "metric": "draft eps-evals/sec (slot evaluations of the batched DiT pass over the whole drf_sample call)",
        "value": evals * args.steps / dt,
        "unit": "eps-evals/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "ms_per_sample": ms_step / B,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if dit["dtype"] == I.BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": "config %d: %s, %d-step %s, %s n=%d, batch %d, guidance %s" % (
            args.config, cfg["name"], S,
            ["DDIM eta=%g" % args.eta if args.eta else "DDIM", "DDPM skip", "Euler shift=%g" % args.shift][args.sampler],
            "aggressive" if mode else "conservative", n, B, cfg["guidance"]),
            "slots_per_full_pass": n * g * B, "evals_per_step": evals},
        "achieved_tflops_whole_call": flops_call / (ms_step * 1e-3) / 1e12,
        "frac_of_bf16_mfma_peak_whole_call": flops_call / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
    }

    if not args.no_roofline:
        # one more call with per-launch HIP events on the library's stream
        den.profile_enable(True)
        step()
        fam = {k: den.profile_read(v) for k, v in (("gemm", drf.PROF_GEMM), ("attn", drf.PROF_ATTN),
                                                    ("elementwise", drf.PROF_ELEMWISE), ("update", drf.PROF_UPDATE))}
        den.profile_enable(False)
        gm = fam["gemm"]
        ach = gm["work"] / (gm["ms"] * 1e-3) / 1e12 if gm["ms"] > 0 else 0.0
        result["roofline"] = {"bound": "mfma", "kernel": "gemm_bf16_xl_kernel (all bf16 GEMM launches of one drf_sample call)",
                              "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                              "frac": ach / PEAK_BF16_TFLOPS,
                              "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH.get(args.config) if default_workload else None,
                              "launches": gm["launches"], "avg_launch_us": gm["ms"] * 1e3 / max(gm["launches"], 1),
                              "flops_per_launch": gm["work"] / max(gm["launches"], 1)}
        result["families_ms"] = {k: round(v["ms"], 3) for k, v in fam.items()}
        at = fam["attn"]
        if at["ms"] > 0:
            result["attn_tflops"] = at["work"] / (at["ms"] * 1e-3) / 1e12
        up = fam["update"]
        if up["ms"] > 0:
            result["update_kernel"] = {"launches": up["launches"], "avg_launch_us": up["ms"] * 1e3 / up["launches"],
                                       "achieved_GBps": up["work"] / (up["ms"] * 1e-3) / 1e9}
        # the update kernel at a size where bandwidth, not launch latency, decides: 4096 samples of this latent,
        # 4 drafts by skip transition (reads x and eps once, writes 4 fields)
        E = dit["in_ch"] * dit["lat_h"] * dit["lat_w"]
        big = 4096
        xb = torch.randn((big, E), device="cuda")
        eb = torch.randn((big, E), device="cuda")
        ob = torch.empty((4, big, E), device="cuda")
        targets = [S - 1, S - 2, S - 3, S - 4] if S >= 5 else [0] * 4
        sd0 = cfg["sched"]
        drf.skip_transition(sd0, xb, eb, S, targets, out=ob)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            drf.skip_transition(sd0, xb, eb, S, targets, out=ob)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 100.0
        result["update_kernel_scaled"] = {"batch": big, "bytes_per_launch": 6 * big * E * 4, "us_per_launch": us,
                                          "achieved_GBps": 6 * big * E * 4 / (us * 1e-6) / 1e9, "peak_GBps": PEAK_HBM_GBS}
        # the same launch with variance: each of the 4 drafts adds its own generated normal field (no extra bytes)
        sdn = dict(cfg["sched"], eta=1.0)
        drf.skip_transition_noise(sdn, xb, eb, S, targets, seed=args.seed, out=ob)
        e0.record()
        for _ in range(10):
            drf.skip_transition_noise(sdn, xb, eb, S, targets, seed=args.seed, out=ob)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 100.0
        result["update_kernel_scaled_noise"] = {"batch": big, "bytes_per_launch": 6 * big * E * 4, "us_per_launch": us,
                                                "achieved_GBps": 6 * big * E * 4 / (us * 1e-6) / 1e9,
                                                "normals_per_s": 4 * big * E / (us * 1e-6)}
        del xb, eb, ob
    den.close()

    if not args.no_cpu_baseline:
        # the oracle as it stands, on a bounded sample of the same work: slot evaluations of the same DiT,
        # one to size the sample, then as many more (in one call, at most 64) as bring it to ~12 s
        from oracle.ref import Oracle
        orc = Oracle(64)
        wd = orc.prepare_weights(w)

        def timed(ns):
            xs = I.latent_noise(dit, ns, args.config)
            cs = I.conditioning(dit, ns, args.config)
            ts = np.linspace(999, 0, ns).astype(np.int32)
            t0 = time.perf_counter()
            orc.dit_eps(dit, wd, xs, ts, cs)
            return time.perf_counter() - t0

        n_done, ct = 1, timed(1)
        more = min(64, int(12.0 / max(ct, 1e-3)))
        if more >= 1 and ct < 10.0:
            ct += timed(more)
            n_done += more
        result["cpu_baseline"] = {"value": n_done / ct, "unit": "eps-evals/s", "cores": orc.threads(), "kind": "oracle",
                                  "sample": "%d slot evaluations of the same DiT (fp64 oracle, %.1f s); a full call is %d of them"
                                            % (n_done, ct, evals)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
