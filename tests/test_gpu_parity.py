"""Parity of the HIP path (through the C ABI) with the CPU oracle on the same seeded
inputs.  Tolerances are the workload's: plan/timestep bookkeeping bit-exact (checked
on the host in test_host_abi.py), fp32 path max-norm relative error <= 1e-4, bf16
path <= 2e-2, where error = max|gpu - oracle| / max|oracle| per sample; the same numbers
also bound every element's error against |oracle| + rms(oracle) (tests/parity.py)."""
import os

import numpy as np
import pytest

from paper_2603_25872_amd import inputs as I
from parity import TOL_BF16, TOL_F32, check, relerr

pytestmark = pytest.mark.gpu


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


SCHED20 = dict(train_steps=1000, beta_start=1e-4, beta_end=0.02, steps=20, eta=0.0)


# ------------------------------------------------------------ update kernels

@pytest.mark.parametrize("shape", [(1, 4, 16, 16), (3, 1021), (2, 4, 32, 32), (5, 3)])
def test_skip_transition_matches_oracle(torch, drf, orc, shape):
    rng = np.random.default_rng(1)
    x = rng.standard_normal(shape).astype(np.float32)
    e = rng.standard_normal(shape).astype(np.float32)
    for s_from, targets in [(20, [19, 18, 17]), (7, [6]), (3, [2, 1, 0]), (5, [9, 5])]:
        got = drf.skip_transition(SCHED20, dev(torch, x), dev(torch, e), s_from, targets).cpu().numpy()
        for j, s_to in enumerate(targets):
            want = orc.skip(x, e, orc.abar_at(SCHED20, s_from), orc.abar_at(SCHED20, s_to))
            assert relerr(got[j], want) < 1e-5, (s_from, s_to)


def test_refine_step_is_the_unit_skip_bit_for_bit(torch, drf, orc):
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 4, 16, 16)).astype(np.float32)
    e = rng.standard_normal((2, 4, 16, 16)).astype(np.float32)
    xd, ed = dev(torch, x), dev(torch, e)
    for s in (20, 11, 1):
        a = drf.refine_step(SCHED20, xd, ed, s).cpu().numpy()
        b = drf.skip_transition(SCHED20, xd, ed, s, [s - 1]).cpu().numpy()[0]
        assert np.array_equal(a, b)
        assert relerr(a, orc.skip(x, e, orc.abar_at(SCHED20, s), orc.abar_at(SCHED20, s - 1))) < 1e-5
    # in-place refine
    y = xd.clone()
    drf.refine_step(SCHED20, y, ed, 9, out=y)
    assert np.array_equal(y.cpu().numpy(), drf.refine_step(SCHED20, xd, ed, 9).cpu().numpy())


def test_update_edge_cases(torch, drf):
    empty = torch.empty((0, 16), dtype=torch.float32, device="cuda")
    assert drf.skip_transition(SCHED20, empty, empty, 5, [4]).shape == (1, 0, 16)
    x = torch.ones((1, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(drf.DrfError):
        drf.skip_transition(SCHED20, x, x, 21, [3])
    with pytest.raises(drf.DrfError):
        drf.skip_transition(SCHED20, x, x, 5, [-1])
    with pytest.raises(drf.DrfError):
        drf.refine_step(dict(SCHED20, eta=1.0), x, x, 5)
    # many targets (more than one argument block)
    tg = [i % 21 for i in range(70)]
    out = drf.skip_transition(SCHED20, x, x * 0.5, 10, tg)
    assert out.shape == (70, 1, 8)
    assert torch.equal(out[3], out[3 + 21]) and torch.equal(out[10], x)


# ------------------------------------------------------------------ DiT forward

def small_dit(cond, dtype, **kw):
    base = dict(depth=2, hidden=128, heads=4, mlp_ratio=4, patch=2, in_ch=4, lat_h=10, lat_w=6, dtype=dtype,
                cond=cond, cond_dim={0: 24, 1: 10, 2: 64}[cond], ctx_len=7 if cond == I.COND_TEXT else 0)
    base.update(kw)
    return base


def make_cond(dit, slots, seed):
    rng = np.random.default_rng(seed)
    if dit["cond"] == I.COND_VECTOR:
        return rng.standard_normal((slots, dit["cond_dim"])).astype(np.float32)
    if dit["cond"] == I.COND_CLASS:
        return rng.integers(0, dit["cond_dim"] + 1, size=slots).astype(np.int32)
    return rng.standard_normal((slots, dit["ctx_len"], dit["cond_dim"])).astype(np.float32)


def check_forward(torch, drf, orc, dit, init, slots, tol, seed=0, trace=True):
    w = I.weights(dit, 40 + seed, init)
    rng = np.random.default_rng(50 + seed)
    x = rng.standard_normal((slots, dit["in_ch"], dit["lat_h"], dit["lat_w"])).astype(np.float32)
    t = rng.integers(0, 1000, size=slots).astype(np.int32)
    t[0], t[-1] = 0, 999
    cond = make_cond(dit, slots, 60 + seed)
    den = drf.Denoiser(dit, w)
    xd, td, cd = dev(torch, x), dev(torch, t), dev(torch, cond)
    errs = {}
    if trace:
        for k in range(dit["depth"] + 1):
            got = den.eps_trace(xd, td, cd, k).cpu().numpy()
            errs["resid%d" % k] = check(got, orc.dit_eps(dit, w, x, t, cond, stop_blocks=k), tol, "resid%d" % k)[0]
    got = den.eps_batched(xd, td, cd).cpu().numpy()
    want = orc.dit_eps(dit, w, x, t, cond)
    errs["eps"] = check(got, want, tol, "eps")[0]
    den.close()
    return errs


@pytest.mark.parametrize("cond", [I.COND_VECTOR, I.COND_CLASS, I.COND_TEXT])
@pytest.mark.parametrize("init", ["paper", "loud"])
def test_fp32_forward_matches_oracle(torch, drf, orc, cond, init):
    check_forward(torch, drf, orc, small_dit(cond, I.F32), init, slots=3, tol=TOL_F32, seed=cond)


def test_fp32_forward_odd_shapes(torch, drf, orc):
    # hidden 72 with 3 heads of 24, one token row, patch 1
    dit = small_dit(I.COND_CLASS, I.F32, hidden=72, heads=3, patch=1, lat_h=3, lat_w=5, depth=1, mlp_ratio=2)
    check_forward(torch, drf, orc, dit, "loud", slots=5, tol=TOL_F32, seed=7)


@pytest.mark.parametrize("cond", [I.COND_VECTOR, I.COND_CLASS, I.COND_TEXT])
@pytest.mark.parametrize("init", ["paper", "loud"])
def test_bf16_forward_matches_oracle(torch, drf, orc, cond, init):
    # 15 tokens per slot: ragged against every tile size; head dim 32
    check_forward(torch, drf, orc, small_dit(cond, I.BF16), init, slots=3, tol=TOL_BF16, seed=10 + cond)


@pytest.mark.parametrize("hidden,heads,lat", [(576, 8, (18, 14)), (384, 6, (32, 32)), (192, 2, (8, 8)), (128, 1, (4, 2))])
def test_bf16_forward_head_dims_and_tiles(torch, drf, orc, hidden, heads, lat):
    # head dims 72, 64, 96, 128->rejected below; 63 / 256 / 16 / 2 tokens per slot
    dit = small_dit(I.COND_CLASS, I.BF16, hidden=hidden, heads=heads, lat_h=lat[0], lat_w=lat[1], depth=2)
    if hidden // heads > 96:
        with pytest.raises(drf.DrfError):
            drf.Denoiser(dit, I.weights(dit, 1))
        return
    check_forward(torch, drf, orc, dit, "loud", slots=5, tol=TOL_BF16, seed=20 + heads)


def test_bf16_text_cross_attention_77(torch, drf, orc):
    dit = small_dit(I.COND_TEXT, I.BF16, hidden=576, heads=8, lat_h=12, lat_w=12, depth=2, cond_dim=128, ctx_len=77)
    check_forward(torch, drf, orc, dit, "loud", slots=2, tol=TOL_BF16, seed=31)


def test_bf16_attention_with_more_work_items_than_cus(torch, drf, orc):
    # launches whose (query block, head, slot) items outnumber the CUs run persistent workgroups:
    # self-attention over a ragged 200-token sequence, and cross-attention of 1024 queries (four
    # query blocks per head) against a 77-row context
    dit = small_dit(I.COND_CLASS, I.BF16, depth=1, lat_h=20, lat_w=40)
    check_forward(torch, drf, orc, dit, "loud", slots=70, tol=TOL_BF16, seed=41, trace=False)
    dit = small_dit(I.COND_TEXT, I.BF16, depth=1, lat_h=64, lat_w=64, ctx_len=77)
    check_forward(torch, drf, orc, dit, "loud", slots=17, tol=TOL_BF16, seed=42, trace=False)


def test_eps_batched_edge_cases(torch, drf):
    dit = small_dit(I.COND_CLASS, I.F32, depth=1)
    den = drf.Denoiser(dit, I.weights(dit, 2))
    x = torch.zeros((0, 4, 10, 6), dtype=torch.float32, device="cuda")
    t = torch.zeros((0,), dtype=torch.int32, device="cuda")
    assert den.eps_batched(x, t, t).shape == (0, 4, 10, 6)
    x1 = torch.randn((2, 4, 10, 6), dtype=torch.float32, device="cuda")
    t1 = torch.tensor([5, 5], dtype=torch.int32, device="cuda")
    # out-of-range class ids are clamped to the null class
    a = den.eps_batched(x1, t1, torch.tensor([10, 10], dtype=torch.int32, device="cuda"))
    b = den.eps_batched(x1, t1, torch.tensor([99, -3], dtype=torch.int32, device="cuda"))
    assert torch.equal(a, b)
    # deterministic: same inputs, same bits; slot order does not matter
    c = den.eps_batched(x1.flip(0).contiguous(), t1, torch.tensor([10, 10], dtype=torch.int32, device="cuda"))
    assert torch.equal(a, c.flip(0))
    with pytest.raises(drf.DrfError):
        drf.Denoiser(dit, I.weights(dit, 2)[:-1])
    den.close()


# ------------------------------------------------------------------ whole path

def run_sample(torch, drf, orc, cfg, tol, mode=None, n=None, batch=None, init="paper", seed=0):
    dit, sd = cfg["dit"], cfg["sched"]
    mode = cfg["mode"] if mode is None else mode
    n = cfg["n"] if n is None else n
    batch = cfg["batch"] if batch is None else batch
    w = I.weights(dit, 70 + seed, init)
    xT = I.latent_noise(dit, batch, 70 + seed)
    cond = I.conditioning(dit, batch, 70 + seed)
    null = I.conditioning(dit, batch, 70 + seed, null=True) if cfg["guidance"] else None
    den = drf.Denoiser(dit, w)
    got = den.sample(sd, mode, n, dev(torch, xT), dev(torch, cond), None if null is None else dev(torch, null),
                     cfg["guidance"] or 0.0).cpu().numpy()
    den.close()
    want = orc.sample_dit(dit, w, sd, mode, n, xT, cond, null, cfg["guidance"] or 0.0)
    return check(got, want, tol, "x_0 %s" % cfg["name"])[0]


@pytest.mark.parametrize("mode", [I.CONSERVATIVE, I.AGGRESSIVE])
@pytest.mark.parametrize("n", [1, 2, 3, 20])
def test_sample_config1_fp32(torch, drf, orc, mode, n):
    # configuration 1 as specified (tiny fp32 DiT, 20-step DDIM), all block sizes incl. n > remaining steps
    run_sample(torch, drf, orc, I.config(1), TOL_F32, mode=mode, n=n)


def test_sample_config1_fp32_loud_with_guidance(torch, drf, orc):
    cfg = I.config(1)
    cfg["guidance"] = 3.0
    run_sample(torch, drf, orc, cfg, TOL_F32, batch=2, init="loud", seed=1)


@pytest.mark.parametrize("mode", [I.CONSERVATIVE, I.AGGRESSIVE])
def test_sample_config2_shape_bf16_reduced(torch, drf, orc, mode):
    # DiT-S width and head count on a 16x16 latent, 3 blocks, 10 steps: the oracle finishes in seconds
    cfg = I.config(2, depth=3, lat_h=16, lat_w=16)
    cfg["sched"]["steps"] = 10
    run_sample(torch, drf, orc, cfg, TOL_BF16, mode=mode, n=3, batch=2)


def test_sample_bf16_guidance_head72(torch, drf, orc):
    # DiT-XL head width (72) and guidance, narrow and shallow
    cfg = I.config(3, depth=2, hidden=576, heads=8, lat_h=8, lat_w=8)
    cfg["sched"]["steps"] = 9
    run_sample(torch, drf, orc, cfg, TOL_BF16, n=4, batch=2)
    run_sample(torch, drf, orc, cfg, TOL_BF16, mode=I.AGGRESSIVE, n=4, batch=2, init="loud", seed=3)


def test_sample_config3_full_depth_against_the_stored_oracle_sample(torch, drf):
    """Configuration 3 exactly as benchmarked except for the batch (1 instead of 8: samples are
    independent): 28 blocks, 50-step DDIM, conservative n = 4, guidance 4.  The expected x_0 was written by
    tests/golden/make_cfg3_sample.py, which calls the CPU oracle only (about half an hour on 8 cores, so
    it is stored instead of recomputed)."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "cfg3_batch1_x0.txt")
    cfg = I.config(3)
    dit, sd = cfg["dit"], cfg["sched"]
    want = np.loadtxt(path).reshape(1, dit["in_ch"], dit["lat_h"], dit["lat_w"])
    w = I.weights(dit, 3)
    xT, cond, null = I.latent_noise(dit, 1, 3), I.conditioning(dit, 1, 3), I.conditioning(dit, 1, 3, null=True)
    den = drf.Denoiser(dit, w)
    got = den.sample(sd, cfg["mode"], cfg["n"], dev(torch, xT), dev(torch, cond), dev(torch, null), cfg["guidance"]).cpu().numpy()
    den.close()
    check(got, want, TOL_BF16, "cfg3 batch 1 x_0")


def test_sample_bf16_text_guidance(torch, drf, orc):
    cfg = I.config(4, depth=2, hidden=192, heads=3, lat_h=8, lat_w=8, cond_dim=64, ctx_len=9)
    cfg["sched"]["steps"] = 7
    run_sample(torch, drf, orc, cfg, TOL_BF16, batch=2, init="loud", seed=4)


def test_sample_equals_manual_loop_over_the_plan(torch, drf, orc):
    """The fused loop against its parts: replay the oracle's plan table with separate
    eps_batched / skip_transition / refine_step calls.  Holds at any size."""
    cfg = I.config(2, depth=2, lat_h=16, lat_w=16)
    cfg["sched"]["steps"] = 11
    dit, sd = cfg["dit"], cfg["sched"]
    B = 2
    w = I.weights(dit, 5)
    den = drf.Denoiser(dit, w)
    xT = dev(torch, I.latent_noise(dit, B, 5))
    cond = dev(torch, I.conditioning(dit, B, 5))
    for mode in (I.CONSERVATIVE, I.AGGRESSIVE):
        got = den.sample(sd, mode, 3, xT, cond)
        rows = orc.plan(sd, mode, 3)
        X, NA, ND = {sd["steps"]: xT}, {}, {}       # refined states, anchor noises, draft noises

        def eps_at(state, tau):
            return den.eps_batched(state, torch.full((B,), tau, dtype=torch.int32, device="cuda"), cond)

        for _, kind, s_from, s_to, tau in rows.tolist():
            if kind == 0:
                NA[s_from] = eps_at(X[s_from], tau)
            elif kind == 1:
                anchor_noise = NA[s_from] if s_from in NA else ND[s_from]
                d = drf.skip_transition(sd, X[s_from], anchor_noise, s_from, [s_to])[0]
                if tau >= 0:
                    ND[s_to] = eps_at(d, tau)
                if s_from - s_to == 1:
                    X[s_to] = d
            else:
                X[s_to] = drf.refine_step(sd, X[s_from], ND[s_from] if s_from in ND else NA[s_from], s_from)
        x = X[0]
        assert relerr(got.cpu().numpy(), x.cpu().numpy()) < 1e-6, mode
    den.close()


def test_sample_edge_cases(torch, drf):
    dit = small_dit(I.COND_CLASS, I.F32, depth=1)
    den = drf.Denoiser(dit, I.weights(dit, 2))
    x = torch.randn((2, 4, 10, 6), dtype=torch.float32, device="cuda")
    c = torch.tensor([1, 2], dtype=torch.int32, device="cuda")
    sd = dict(SCHED20, steps=4)
    a = den.sample(sd, I.CONSERVATIVE, 100, x, c)            # n beyond S
    b = den.sample(sd, I.CONSERVATIVE, 4, x, c)
    assert torch.equal(a, b)
    one = den.sample(dict(SCHED20, steps=1), I.AGGRESSIVE, 3, x, c)
    assert torch.isfinite(one).all()
    y = x.clone()
    den.sample(sd, I.AGGRESSIVE, 2, y, c, out=y)             # in place
    assert torch.equal(y, den.sample(sd, I.AGGRESSIVE, 2, x, c))
    for bad in (dict(n=0), dict(mode=3)):
        with pytest.raises(drf.DrfError):
            den.sample(sd, bad.get("mode", 0), bad.get("n", 2), x, c)
    empty = torch.empty((0, 4, 10, 6), dtype=torch.float32, device="cuda")
    assert den.sample(sd, 0, 2, empty, c[:0]).shape == (0, 4, 10, 6)
    den.close()


@pytest.mark.parametrize("steps,batch,guidance", [(50, 24, 3.0), (100, 2, None)])
def test_sample_with_more_conditioning_rows_than_one_chunk_or_flush(torch, drf, orc, steps, batch, guidance):
    """The modulation rows of a call are produced per chunk of passes (at most 1024 rows unless one pass has more)
    and per flush of 64 timestep groups: 50 steps x 48 slot rows = 2400 rows make three chunks, and 100 steps at
    batch 2 make one chunk of two flushes.  Tiny fp32 DiT of configuration 1, aggressive n = 3, against the oracle."""
    cfg = I.config(1)
    cfg["sched"]["steps"] = steps
    cfg["guidance"] = guidance
    run_sample(torch, drf, orc, cfg, TOL_F32, mode=I.AGGRESSIVE, n=3, batch=batch, seed=8)
