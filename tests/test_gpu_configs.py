"""Parity at the stated shapes of the workload configurations (BASELINE configurations 2-5), in the launch
configuration bench.py times.  Expected values are stored under tests/golden/, written by scripts that
call the CPU oracle only (make_cfg2_sample.py, make_cfg3_sample.py, make_pass_goldens.py): the oracle
needs minutes per slot at these sizes."""
import os

import numpy as np
import pytest

from paper_2603_25872_amd import inputs as I
from parity import TOL_BF16, check, relerr

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "GPU tests need a GPU"
    return t


@pytest.fixture(scope="module")
def drf():
    from paper_2603_25872_amd import drf as d
    d.lib()
    return d


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def load_pass_golden(idx):
    """records of tests/golden/cfg{idx}_pass.txt: name -> (values, max|v| and rms of the whole field)"""
    recs, name = {}, None
    for line in open(os.path.join(GOLDEN, "cfg%d_pass.txt" % idx)):
        if line.startswith("#"):
            f = line.split()
            if len(f) > 2 and f[2] == "count":
                name = f[1]
                recs[name] = ([], float(f[5]), float(f[7]))
            continue
        recs[name][0].append(float(line))
    return {k: (np.array(v[0]), v[1], v[2]) for k, v in recs.items()}


def first_draft_taus(drf, cfg):
    rows = drf.plan_build(cfg["sched"], cfg["mode"], cfg["n"]).tolist()
    first = min(r[0] for r in rows if r[1] == 1)
    return [r[4] for r in rows if r[0] == first and r[1] == 1 and r[4] >= 0]


def test_config2_as_specified_against_the_stored_oracle_sample(torch, drf):
    """Configuration 2 exactly as stated: 12 blocks, hidden 384, 32x32 latent, 50-step DDIM, aggressive n = 3,
    batch 4 (Algorithm 1)."""
    cfg = I.config(2)
    dit, sd, B = cfg["dit"], cfg["sched"], cfg["batch"]
    want = np.loadtxt(os.path.join(GOLDEN, "cfg2_x0.txt")).reshape(B, dit["in_ch"], dit["lat_h"], dit["lat_w"])
    den = drf.Denoiser(dit, I.weights(dit, 2))
    got = den.sample(sd, cfg["mode"], cfg["n"], dev(torch, I.latent_noise(dit, B, 2)), dev(torch, I.conditioning(dit, B, 2)))
    got = got.cpu().numpy()
    den.close()
    check(got, want, TOL_BF16, "cfg2 x_0")


@pytest.mark.parametrize("idx", [3, 4, 5])
def test_full_draft_pass_at_the_stated_shape(torch, drf, idx):
    """One full draft pass (every draft group with its own timestep, cond and null halves) of configurations
    3 (64 slots x 256 tokens), 4 (6 slots x 4096 tokens, 77 x 1024 text context, cross-attention) and 5 (64 slots
    x 1024 tokens, 8 distinct timesteps), as drf_sample launches it.  With the test-only loud initialisation the
    residual stream after block 1 and after the last block and eps are compared with the oracle on sampled slots
    at seeded positions; with the workload's own initialisation, eps."""
    cfg = I.config(idx)
    dit = cfg["dit"]
    gold = load_pass_golden(idx)
    taus = first_draft_taus(drf, cfg)
    x, t, cond = I.draft_pass(idx, taus)
    slots = x.shape[0]
    assert slots == cfg["n"] * (2 if cfg["guidance"] else 1) * cfg["batch"]
    T = (dit["lat_h"] // dit["patch"]) * (dit["lat_w"] // dit["patch"])
    rsz, esz = T * dit["hidden"], dit["in_ch"] * dit["lat_h"] * dit["lat_w"]
    xd, td, cd = dev(torch, x), dev(torch, t), dev(torch, cond)
    seen = 0
    for init in ("loud", "paper"):
        den = drf.Denoiser(dit, I.weights(dit, idx, init))
        out = {}
        if init == "loud":
            out["resid1"] = den.eps_trace(xd, td, cd, 1)
            out["residL"] = den.eps_trace(xd, td, cd, dit["depth"])
        out["eps"] = den.eps_batched(xd, td, cd)
        for what, val in out.items():
            assert bool(torch.isfinite(val).all()), (init, what)
            for name, (want, vmax, rms) in gold.items():
                i, w, s = name.split(".")
                if i != init or w != what:
                    continue
                s = int(s[4:])
                pts = I.sample_points(want.size, rsz if what.startswith("resid") else esz, idx * 100 + s)
                got = val[s].reshape(-1)[torch.from_numpy(pts).cuda()].cpu().numpy()
                check(got, want, TOL_BF16, "cfg%d %s" % (idx, name), scale=vmax, rms=rms)
                seen += 1
        # the device path is deterministic: a second run gives the same bits
        assert torch.equal(out["eps"], den.eps_batched(xd, td, cd)), init
        den.close()
    assert seen == len(gold)


def test_config3_sample_at_the_benchmarked_batch(torch, drf):
    """drf_sample of configuration 3 exactly as benchmarked (batch 8: 64-slot draft passes, 16-slot stand-alone
    passes).  Sample 0 has the inputs of the stored batch-1 oracle sample; every sample must also agree with a
    batch-1 call on its own inputs (samples are independent; tile shapes differ between the two batch sizes,
    so the agreement is to rounding, not bit for bit)."""
    cfg = I.config(3)
    dit, sd, B = cfg["dit"], cfg["sched"], cfg["batch"]
    want0 = np.loadtxt(os.path.join(GOLDEN, "cfg3_batch1_x0.txt")).reshape(1, dit["in_ch"], dit["lat_h"], dit["lat_w"])
    xT, cond, null = I.latent_noise(dit, B, 3), I.conditioning(dit, B, 3), I.conditioning(dit, B, 3, null=True)
    den = drf.Denoiser(dit, I.weights(dit, 3))
    got = den.sample(sd, cfg["mode"], cfg["n"], dev(torch, xT), dev(torch, cond), dev(torch, null), cfg["guidance"])
    check(got[:1].cpu().numpy(), want0, TOL_BF16, "cfg3 batch 8, sample 0")
    assert torch.equal(got, den.sample(sd, cfg["mode"], cfg["n"], dev(torch, xT), dev(torch, cond), dev(torch, null), cfg["guidance"]))
    for b in (3, 7):
        one = den.sample(sd, cfg["mode"], cfg["n"], dev(torch, xT[b:b + 1]), dev(torch, cond[b:b + 1]), dev(torch, null[b:b + 1]),
                         cfg["guidance"])
        e = relerr(got[b:b + 1].cpu().numpy(), one.cpu().numpy())
        print("cfg3 batch 8 sample %d vs its batch-1 call: %.3e" % (b, e), flush=True)
        assert e < 5e-3, (b, e)
    den.close()


def test_bf16_determinism_on_the_split_k_and_persistent_paths(torch, drf):
    """Two runs, same bits, on the 16-slot pass of configuration 3 (out-proj / fc2 take the tile that splits K
    between two wave groups) and on its 64-slot pass (persistent attention workgroups)."""
    cfg = I.config(3, depth=2)
    dit = cfg["dit"]
    den = drf.Denoiser(dit, I.weights(dit, 3, "loud"))
    rng = np.random.default_rng(5)
    for slots in (16, 64):
        x = dev(torch, rng.standard_normal((slots, 4, 32, 32)).astype(np.float32))
        t = dev(torch, rng.integers(0, 1000, slots).astype(np.int32))
        c = dev(torch, rng.integers(0, 1001, slots).astype(np.int32))
        a = den.eps_batched(x, t, c)
        for _ in range(3):
            assert torch.equal(a, den.eps_batched(x, t, c)), slots
    den.close()


def test_config2_shape_under_the_other_samplers(torch, drf):
    """Configuration 2 at its stated shape under stochastic DDIM (eta = 0.5), the DDPM posterior skip (both with
    the library's in-kernel noise stream, which the oracle drew with its own generator) and the Euler skip with
    time shift 3, against stored oracle samples (tests/golden/make_cfg2_samplers.py)."""
    cfg = I.config(2)
    dit, B = cfg["dit"], cfg["batch"]
    recs, name = {}, None
    for line in open(os.path.join(GOLDEN, "cfg2_samplers_x0.txt")):
        if line.startswith("#"):
            f = line.split()
            if len(f) == 4 and f[2] == "sample":
                name = (f[1], int(f[3]))
                recs[name] = []
            continue
        recs[name].append(float(line))
    assert len(recs) == 6
    den = drf.Denoiser(dit, I.weights(dit, 2))
    xT, cond = dev(torch, I.latent_noise(dit, B, 2)), dev(torch, I.conditioning(dit, B, 2))
    for sname, extra in (("ddim_eta0.5", dict(eta=0.5)), ("ddpm", dict(sampler=1)), ("euler_shift3", dict(sampler=2, shift=3.0))):
        sd = dict(cfg["sched"], **extra)
        if extra.get("sampler") == 2:
            got = den.sample(sd, cfg["mode"], cfg["n"], xT, cond)
        else:
            got = den.sample_noise(sd, cfg["mode"], cfg["n"], xT, cond, seed=4242, field0=0)
        got = got.cpu().numpy()
        for b in (0, 3):
            want = np.array(recs[(sname, b)]).reshape(got[b].shape)
            check(got[b][None], want[None], TOL_BF16, "cfg2 %s sample %d" % (sname, b))
    den.close()
