"""Throughput of the DRiffusion hot path on one MI355X.

One "step" is one drf_sample call: the whole draft-and-refine loop (all S sampling
steps: batched DiT passes + fused guidance/refine/draft updates) over one batch of
synthetic latents, inputs resident in HBM.  Default workload: configuration 3
(DiT-XL/2-shaped, bf16, guidance 4, 50-step DDIM, conservative n=4, batch 8).

Prints ONE JSON line: eps-evals/s over the whole call, ms per step; `roofline`: the full draft pass
(all kernels of one batched predictor pass over the n draft groups: its algorithmic flops over its
duration, measured with HIP events on the library's stream inside drf_sample during an extra
instrumented call), with the bf16 GEMM launches alone as the sub-key `gemm`, the spec peak as `peak`
and what this GPU delivers for an MFMA-only loop and a plain copy as `peak_measured`; and
`cpu_baseline`: the CPU oracle timed on a bounded sample of the same workload (slot evaluations of
the same DiT).  `--calibrate` prints only the measured ceilings."""
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
# HBM-side bytes of the default workload from rocprofv3 --pmc runs (FETCH_SIZE and WRITE_SIZE, each scaled by what
# the same counter reads for a plain 1 GiB copy; profiles/drf_sample_cfg3_pmc_traffic_mfma.txt): per full draft pass
# (all kernels of one 64-slot pass) and per bf16 GEMM launch on average.  Counters cannot be read inside this
# process, so these are the committed profile's figures and only reported for the workload they were measured on.
PASS_TRAFFIC_BYTES = {3: 4.73e10}
GEMM_TRAFFIC_BYTES_PER_LAUNCH = {3: 1.873e8}


def calibrate(torch, drf):
    """What this GPU delivers for a loop of nothing but the GEMM kernel's MFMA instruction (random and constant
    operands: the clock depends on operand toggling) and for a plain 1 GiB copy kernel."""
    out = {"mfma_bf16_random_operands_TFLOPs": max(drf.calibrate_mfma_bf16(True, 5) for _ in range(2)),
           "mfma_bf16_constant_operands_TFLOPs": max(drf.calibrate_mfma_bf16(False, 5) for _ in range(2))}
    a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    b = torch.empty_like(a)
    out["copy_1GiB_GBps"] = max(drf.calibrate_copy(a, b, 5) for _ in range(2))
    del a, b
    # The library's own wide-tile GEMM on the MLP out-projection shape of configuration 3 (16384 x 1152 x 4608),
    # back-to-back launches, with N(0, 1) x N(0, 0.02) operands and with all-zero operands: the same instruction
    # stream, so the ratio is what the chip's power management takes for the operands' bit toggling.
    M, N, K = 16384, 1152, 4608

    def gemm_rate(A, W, iters=20):
        bias = torch.zeros(N, device="cuda")
        o = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        for _ in range(3):
            drf.probe_gemm_bf16(A, W, bias, out=o)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(iters):
            drf.probe_gemm_bf16(A, W, bias, out=o)
        e1.record()
        torch.cuda.synchronize()
        return 2.0 * M * N * K * iters / (e0.elapsed_time(e1) * 1e-3) / 1e12

    out["gemm_16384x1152x4608_zero_operands_TFLOPs"] = gemm_rate(torch.zeros((M, K), dtype=torch.bfloat16, device="cuda"),
                                                                  torch.zeros((N, K), dtype=torch.bfloat16, device="cuda"))
    out["gemm_16384x1152x4608_random_operands_TFLOPs"] = gemm_rate(
        torch.randn((M, K), device="cuda").to(torch.bfloat16), (torch.randn((N, K), device="cuda") * 0.02).to(torch.bfloat16))
    return out


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
    ap.add_argument("--graphs", type=int, default=2,
                    help="0: drf_sample launches kernel by kernel; 2 (default): the launch sequence is captured into a HIP graph "
                         "at the first (warm-up) call and replayed; 1: the library's default, capture at the second call")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--n-sweep", action="store_true",
                    help="only time drf_sample at batch 1 (unless --batch is given) for n in 1, 2, 4, 8 in both modes: the one-GPU "
                         "analogue of the paper's latency-versus-devices figure; prints one JSON line with the table")
    ap.add_argument("--calibrate", action="store_true", help="only measure the MFMA-loop and copy-kernel ceilings of this GPU")
    ap.add_argument("--update-probe", action="store_true",
                    help="only run the fused update kernel (guidance, chain of n, n next drafts) at batch 4096: the launch a "
                         "profiler run reads FETCH_SIZE / WRITE_SIZE for")
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
    if args.calibrate:
        print(json.dumps({"peak_measured": calibrate(torch, drf)}))
        return

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

    def update_probe(iters):
        """The fused update kernel as drf_sample launches it after a full draft pass of the aggressive mode (guidance
        combine of n (cond, null) field pairs, chain of n updates, n next drafts) on 4096 samples of this latent."""
        E = dit["in_ch"] * dit["lat_h"] * dit["lat_w"]
        big, nn = max(1, min(4096, (1 << 24) // E)), min(n, 4)
        xb = torch.randn((big, E), device="cuda")
        eb = torch.randn((nn, g, big, E), device="cuda")
        xo = torch.empty_like(xb)
        do = torch.empty((nn, big, E), device="cuda")
        s_from = min(S, 2 * nn + 1)
        nbytes = 4 * big * E * (1 + g * nn + 1 + nn)
        drf.probe_update_fused(cfg["sched"], s_from, nn, nn, g, cfg["guidance"] or 0.0, xb, eb, xo, do)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()                                  # torch's current stream is the stream the library is given
        for _ in range(iters):
            drf.probe_update_fused(cfg["sched"], s_from, nn, nn, g, cfg["guidance"] or 0.0, xb, eb, xo, do)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / iters
        return {"form": "guidance g=%d, chain of %d, %d next drafts" % (g, nn, nn), "batch": big, "bytes_per_launch": nbytes,
                "us_per_launch": us, "achieved_GBps": nbytes / (us * 1e-6) / 1e9, "peak_GBps": PEAK_HBM_GBS}

    if args.update_probe:
        print(json.dumps({"update_kernel_fused_scaled": update_probe(3)}))
        return

    if args.n_sweep:
        Bs = 1 if args.batch is None else args.batch
        den = drf.Denoiser(dit, I.weights(dit, args.config))
        den.use_graphs(args.graphs)
        xs = torch.from_numpy(I.latent_noise(dit, Bs, args.config)).cuda()
        cs = torch.from_numpy(I.conditioning(dit, Bs, args.config)).cuda()
        ns = torch.from_numpy(I.conditioning(dit, Bs, args.config, null=True)).cuda() if cfg["guidance"] else None
        os_ = torch.empty_like(xs)
        table = []
        for m_, mname in ((I.CONSERVATIVE, "conservative"), (I.AGGRESSIVE, "aggressive")):
            for k in (1, 2, 3, 4, 8):
                for _ in range(max(args.warmup, 1)):
                    den.sample(cfg["sched"], m_, k, xs, cs, ns, cfg["guidance"] or 0.0, out=os_)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps):
                    den.sample(cfg["sched"], m_, k, xs, cs, ns, cfg["guidance"] or 0.0, out=os_)
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t0) / args.steps * 1e3
                passes = int(drf.plan_build(cfg["sched"], m_, k)[:, 0].max()) + 1
                table.append({"mode": mname, "n": k, "ms_per_call": ms, "passes": passes, "ideal_speedup": S / passes})
        base = {r["mode"]: r["ms_per_call"] for r in table if r["n"] == 1}
        for r in table:
            r["speedup_vs_n1"] = base[r["mode"]] / r["ms_per_call"]
        den.close()
        print(json.dumps({"n_sweep": {"workload": "config %d: %s, %d-step DDIM, batch %d, guidance %s" % (
            args.config, cfg["name"], S, Bs, cfg["guidance"]), "steps": args.steps, "rows": table}}))
        return

    w = I.weights(dit, args.config)
    den = drf.Denoiser(dit, w)
    den.reserve(n * g * B)
    den.use_graphs(args.graphs)
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
    t_host = time.perf_counter() - t0               # the calls have returned; the GPU is still working
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert bool(torch.isfinite(out).all())
    gstats = den.graph_stats()

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
        "host_ms_per_step_until_return": t_host / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if dit["dtype"] == I.BF16 else "f32",
        "data": "synthetic",
        "graph_replay": {"mode": args.graphs, "calls_replayed": gstats["replays"], "captures_failed": gstats["failed"]},
        "config": {"workload": "config %d: %s, %d-step %s, %s n=%d, batch %d, guidance %s" % (
            args.config, cfg["name"], S,
            ["DDIM eta=%g" % args.eta if args.eta else "DDIM", "DDPM skip", "Euler shift=%g" % args.shift][args.sampler],
            "aggressive" if mode else "conservative", n, B, cfg["guidance"]),
            "slots_per_full_pass": n * g * B, "evals_per_step": evals},
        "achieved_tflops_whole_call": flops_call / (ms_step * 1e-3) / 1e12,
        "frac_of_bf16_mfma_peak_whole_call": flops_call / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
    }

    if not args.no_roofline:
        # call A: each predictor pass of the call bracketed as a whole (two events per pass, kernels undisturbed)
        den.profile_enable(2)
        step()
        pf, po = den.profile_read(drf.PROF_PASS_FULL), den.profile_read(drf.PROF_PASS_OTHER)
        # call B: every launch bracketed, per kernel family
        den.profile_enable(1)
        step()
        fam = {k: den.profile_read(v) for k, v in (("gemm", drf.PROF_GEMM), ("attn", drf.PROF_ATTN),
                                                    ("elementwise", drf.PROF_ELEMWISE), ("update", drf.PROF_UPDATE))}
        den.profile_enable(0)
        peaks = calibrate(torch, drf)
        gm = fam["gemm"]
        g_ach = gm["work"] / (gm["ms"] * 1e-3) / 1e12 if gm["ms"] > 0 else 0.0
        gemm = {"kernel": "gemm_bf16_xl_kernel (all bf16 GEMM launches of one drf_sample call)", "achieved": g_ach,
                "frac": g_ach / PEAK_BF16_TFLOPS, "launches": gm["launches"],
                "avg_launch_us": gm["ms"] * 1e3 / max(gm["launches"], 1), "flops_per_launch": gm["work"] / max(gm["launches"], 1),
                "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH.get(args.config) if default_workload else None}
        dom = pf if pf["launches"] > 0 else po          # n = 1 conservative has no draft pass
        ach = dom["work"] / (dom["ms"] * 1e-3) / 1e12 if dom["ms"] > 0 else 0.0
        result["roofline"] = {"bound": "mfma",
                              "kernel": "full draft pass: all kernels of one batched predictor pass over %d slots (%d per call)"
                                        % (n * g * B if pf["launches"] > 0 else g * B, dom["launches"]),
                              "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
                              "traffic": PASS_TRAFFIC_BYTES.get(args.config) if default_workload else None,
                              "avg_pass_ms": dom["ms"] / max(dom["launches"], 1),
                              "flops_per_pass": dom["work"] / max(dom["launches"], 1),
                              "peak_measured": peaks,
                              "frac_of_measured_mfma_random": ach / peaks["mfma_bf16_random_operands_TFLOPs"],
                              "gemm": gemm}
        if pf["launches"] > 0 and po["launches"] > 0:
            o_ach = po["work"] / (po["ms"] * 1e-3) / 1e12
            result["roofline"]["other_passes"] = {"what": "stand-alone evaluations and cut-short blocks", "passes": po["launches"],
                                                  "avg_pass_ms": po["ms"] / po["launches"], "achieved": o_ach,
                                                  "frac": o_ach / PEAK_BF16_TFLOPS}
        result["families_ms"] = {k: round(v["ms"], 3) for k, v in fam.items()}
        at = fam["attn"]
        if at["ms"] > 0:
            result["attn_tflops"] = at["work"] / (at["ms"] * 1e-3) / 1e12
        up = fam["update"]
        if up["ms"] > 0:
            result["update_kernel"] = {"launches": up["launches"], "avg_launch_us": up["ms"] * 1e3 / up["launches"],
                                       "achieved_GBps": up["work"] / (up["ms"] * 1e-3) / 1e9}
        result["update_kernel_fused_scaled"] = update_probe(10)
        # the update kernel at a size where bandwidth, not launch latency, decides: 4096 samples of this latent,
        # 4 drafts by skip transition (reads x and eps once, writes 4 fields)
        E = dit["in_ch"] * dit["lat_h"] * dit["lat_w"]
        big = max(1, min(4096, (1 << 24) // E))
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
        # one to size the sample, then as many more (in one call, at most 64) as bring it to ~10 s.  The fp64
        # build is the parity authority and the reported baseline; the fp32 build of the same text is timed
        # beside it on a shorter sample.
        from oracle.ref import Oracle

        def timed_oracle(bits, budget):
            orc = Oracle(bits)
            wd = orc.prepare_weights(w)

            def timed(ns):
                xs = I.latent_noise(dit, ns, args.config)
                cs = I.conditioning(dit, ns, args.config)
                ts = np.linspace(999, 0, ns).astype(np.int32)
                t0 = time.perf_counter()
                orc.dit_eps(dit, wd, xs, ts, cs)
                return time.perf_counter() - t0

            n_done, ct = 1, timed(1)
            more = min(64, int(budget / max(ct, 1e-3)))
            if more >= 1 and ct < budget:
                ct += timed(more)
                n_done += more
            return n_done, ct, orc.threads()

        n64, t64, cores = timed_oracle(64, 10.0)
        n32, t32, _ = timed_oracle(32, 5.0)
        result["cpu_baseline"] = {"value": n64 / t64, "unit": "eps-evals/s", "cores": cores, "kind": "oracle",
                                  "precision": "fp64 build (the parity authority)",
                                  "sample": "%d slot evaluations of the same DiT (fp64 oracle, %.1f s); a full call is %d of them"
                                            % (n64, t64, evals),
                                  "fp32_build": {"value": n32 / t32, "sample": "%d slot evaluations, %.1f s" % (n32, t32)}}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
