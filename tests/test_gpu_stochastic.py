"""Parity of the stochastic and Euler samplers of the HIP path with the CPU oracle:
skip transitions with variance (DDIM eta > 0, DDPM posterior), the Euler skip, the
library's counter-based normal stream, and the whole draft-and-refine loop with fresh
noise.  Same tolerances as the deterministic path: fp32 <= 1e-4, bf16 <= 2e-2
(max-norm relative per sample); the explicit-field and generated-field routes of the
kernel must agree bit for bit."""
import numpy as np
import pytest

from paper_2603_25872_amd import inputs as I

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16 = 2e-2
BASE = dict(train_steps=1000, beta_start=1e-4, beta_end=0.02, steps=20)
DDIM, DDPM, EULER = 0, 1, 2


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


def relerr(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    g, w = got.reshape(got.shape[0], -1), want.reshape(want.shape[0], -1)
    return float((np.abs(g - w).max(axis=1) / np.abs(w).max(axis=1)).max())


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# ------------------------------------------------------------- normal stream

@pytest.mark.parametrize("F,fields,field0", [(4096, 3, 0), (1003, 2, 5), (1, 1, 7), (6, 4, 0xfffffff0)])
def test_normal_fill_matches_oracle(torch, drf, orc, F, fields, field0):
    seed = (0x1234 << 32) | 0xdeadbeef
    got = drf.normal_fill(seed, field0, fields, F).cpu().numpy()
    want = orc.normal_fill(seed, field0, fields, F)
    # single-precision log / sincos against double: a few ulp of the radius (<= 5.7)
    assert np.abs(got - want).max() < 4e-6
    assert np.isfinite(got).all()


def test_normal_fill_large_is_standard_normal(torch, drf):
    z = drf.normal_fill(77, 0, 4, 1 << 20).cpu().numpy().ravel().astype(np.float64)
    assert abs(z.mean()) < 3e-3 and abs(z.var() - 1) < 4e-3
    assert abs((z ** 4).mean() - 3) < 3e-2


# ------------------------------------------------------- skips with variance

@pytest.mark.parametrize("shape", [(1, 4, 16, 16), (3, 1021), (5, 3)])
@pytest.mark.parametrize("extra", [dict(eta=1.0), dict(eta=0.3), dict(sampler=DDPM)])
def test_stochastic_skip_matches_oracle(torch, drf, orc, shape, extra):
    sd = dict(BASE, **extra)
    rng = np.random.default_rng(1)
    x = rng.standard_normal(shape).astype(np.float32)
    e = rng.standard_normal(shape).astype(np.float32)
    for s_from, targets in [(20, [19, 18, 17, 12]), (7, [6]), (3, [2, 1, 0]), (5, [5, 4])]:
        z = rng.standard_normal((len(targets),) + shape).astype(np.float32)
        got = drf.skip_transition_noise(sd, dev(torch, x), dev(torch, e), s_from, targets, z=dev(torch, z)).cpu().numpy()
        for j, s_to in enumerate(targets):
            af, at = orc.abar_at(sd, s_from), orc.abar_at(sd, s_to)
            if extra.get("sampler") == DDPM:
                want = orc.ddpm_skip(x, e, z[j], af, at)
            else:
                want = orc.skip_eta(x, e, z[j], af, at, orc.sigma(extra["eta"], af, at))
            assert relerr(got[j], want) < 1e-5, (s_from, s_to)


@pytest.mark.parametrize("shape", [(2, 4, 16, 16), (3, 1021)])
def test_generated_fields_equal_explicit_fields_bit_for_bit(torch, drf, shape):
    # vector (float4) and scalar routes of the kernel both read block q = element / 4 of the field
    sd = dict(BASE, eta=1.0)
    x = torch.randn(shape, dtype=torch.float32, device="cuda")
    e = torch.randn(shape, dtype=torch.float32, device="cuda")
    targets = [19, 17, 11]
    F = x.numel()
    z = drf.normal_fill(2024, 9, len(targets), F).reshape((len(targets),) + tuple(shape))
    a = drf.skip_transition_noise(sd, x, e, 20, targets, z=z)
    b = drf.skip_transition_noise(sd, x, e, 20, targets, seed=2024, field0=9)
    assert torch.equal(a, b)
    c = drf.skip_transition_noise(sd, x, e, 20, targets, seed=2025, field0=9)
    assert not torch.equal(a, c)


def test_euler_skip_matches_oracle(torch, drf, orc):
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 333)).astype(np.float32)
    v = rng.standard_normal((2, 333)).astype(np.float32)
    for shift in (1.0, 3.0):
        sd = dict(BASE, sampler=EULER, shift=shift)
        targets = [19, 15, 0, 20]
        got = drf.skip_transition(sd, dev(torch, x), dev(torch, v), 20, targets).cpu().numpy()
        for j, s_to in enumerate(targets):
            want = orc.euler_skip(x, v, orc.sigma_at(sd, 20), orc.sigma_at(sd, s_to))
            assert relerr(got[j], want) < 1e-6
        # a refine step is the unit skip
        a = drf.refine_step(sd, dev(torch, x), dev(torch, v), 8).cpu().numpy()
        assert relerr(a, orc.euler_skip(x, v, orc.sigma_at(sd, 8), orc.sigma_at(sd, 7))) < 1e-6


def test_stochastic_update_edge_cases(torch, drf):
    x = torch.ones((1, 8), dtype=torch.float32, device="cuda")
    sd = dict(BASE, eta=1.0)
    with pytest.raises(drf.DrfError):
        drf.skip_transition(sd, x, x, 5, [4])                       # variance but no noise source
    with pytest.raises(drf.DrfError):
        drf.skip_transition_noise(sd, x, x, 5, [6], seed=1)          # variance needs a move towards data
    # no variance on the way to index 0 or on the identity jump: no source needed
    out = drf.skip_transition(sd, x, x * 0.25, 5, [0, 5])
    assert torch.equal(out[1], x) and torch.isfinite(out).all()
    empty = torch.empty((0, 16), dtype=torch.float32, device="cuda")
    assert drf.skip_transition_noise(sd, empty, empty, 5, [4], seed=3).shape == (1, 0, 16)
    # more targets than one argument block holds; field numbers follow the target index
    tg = [i % 10 for i in range(70)]
    big = drf.skip_transition_noise(sd, x, x * 0.5, 10, tg, seed=11)
    one = drf.skip_transition_noise(sd, x, x * 0.5, 10, [tg[66]], seed=11, field0=66)
    assert torch.equal(big[66], one[0])


# ------------------------------------------------------------------ whole path

def run_sample(torch, drf, orc, cfg, sd, tol, mode, n, batch, source, init="paper", seed=0):
    dit = cfg["dit"]
    w = I.weights(dit, 170 + seed, init)
    xT = I.latent_noise(dit, batch, 170 + seed)
    cond = I.conditioning(dit, batch, 170 + seed)
    null = I.conditioning(dit, batch, 170 + seed, null=True) if cfg["guidance"] else None
    cnt = orc.noise_count(sd, mode, n)
    assert drf.noise_count(sd, mode, n) == cnt
    den = drf.Denoiser(dit, w)
    args = (sd, mode, n, dev(torch, xT), dev(torch, cond), None if null is None else dev(torch, null),
            cfg["guidance"] or 0.0)
    if source == "explicit":
        z = np.random.default_rng(900 + seed).standard_normal((cnt,) + xT.shape).astype(np.float32)
        got = den.sample_noise(*args, z=dev(torch, z)).cpu().numpy()
    elif source == "stream":
        # the oracle draws the same stream with its own generator
        z = orc.normal_fill(4242 + seed, 3, cnt, xT.size).reshape((cnt,) + xT.shape)
        got = den.sample_noise(*args, seed=4242 + seed, field0=3).cpu().numpy()
    else:
        z = None
        got = den.sample(*args).cpu().numpy()
    den.close()
    want = orc.sample_dit(dit, w, sd, mode, n, xT, cond, null, cfg["guidance"] or 0.0, z=z)
    err = relerr(got, want)
    assert np.isfinite(err) and err < tol, err
    return err


@pytest.mark.parametrize("mode", [I.CONSERVATIVE, I.AGGRESSIVE])
@pytest.mark.parametrize("n", [1, 3, 20])
@pytest.mark.parametrize("extra", [dict(eta=1.0), dict(eta=0.5), dict(sampler=DDPM)])
def test_stochastic_sample_config1_fp32(torch, drf, orc, mode, n, extra):
    cfg = I.config(1)
    sd = dict(cfg["sched"], **extra)
    run_sample(torch, drf, orc, cfg, sd, TOL_F32, mode, n, cfg["batch"], "explicit")


@pytest.mark.parametrize("mode", [I.CONSERVATIVE, I.AGGRESSIVE])
def test_stochastic_sample_from_the_library_stream(torch, drf, orc, mode):
    cfg = I.config(1)
    cfg["guidance"] = 2.5
    sd = dict(cfg["sched"], eta=1.0)
    run_sample(torch, drf, orc, cfg, sd, TOL_F32, mode, 4, 3, "stream", init="loud", seed=1)


@pytest.mark.parametrize("mode", [I.CONSERVATIVE, I.AGGRESSIVE])
@pytest.mark.parametrize("shift", [1.0, 3.0])
def test_euler_sample_config1_fp32(torch, drf, orc, mode, shift):
    cfg = I.config(1)
    sd = dict(cfg["sched"], sampler=EULER, shift=shift)
    run_sample(torch, drf, orc, cfg, sd, TOL_F32, mode, 3, cfg["batch"], None)


def test_stochastic_and_euler_sample_bf16_guidance(torch, drf, orc):
    # DiT-XL head width (72), guidance, narrow and shallow
    cfg = I.config(3, depth=2, hidden=576, heads=8, lat_h=8, lat_w=8)
    base = dict(cfg["sched"], steps=9)
    run_sample(torch, drf, orc, cfg, dict(base, eta=1.0), TOL_BF16, I.CONSERVATIVE, 4, 2, "explicit")
    run_sample(torch, drf, orc, cfg, dict(base, sampler=DDPM), TOL_BF16, I.AGGRESSIVE, 4, 2, "stream", seed=2)
    run_sample(torch, drf, orc, cfg, dict(base, sampler=EULER, shift=3.0), TOL_BF16, I.CONSERVATIVE, 4, 2, None, seed=3)


def test_euler_sample_bf16_text(torch, drf, orc):
    # the flow-matching workload's shape: text context, guidance, shifted sigma grid
    cfg = I.config(4, depth=2, hidden=192, heads=3, lat_h=8, lat_w=8, cond_dim=64, ctx_len=9)
    sd = dict(cfg["sched"], steps=7, sampler=EULER, shift=3.0)
    run_sample(torch, drf, orc, cfg, sd, TOL_BF16, cfg["mode"], cfg["n"], 2, None, init="loud", seed=4)


def test_stochastic_sample_semantics(torch, drf):
    dit = dict(depth=1, hidden=128, heads=4, mlp_ratio=4, patch=2, in_ch=4, lat_h=10, lat_w=6, dtype=I.F32,
               cond=I.COND_CLASS, cond_dim=10, ctx_len=0)
    den = drf.Denoiser(dit, I.weights(dit, 2))
    x = torch.randn((2, 4, 10, 6), dtype=torch.float32, device="cuda")
    c = torch.tensor([1, 2], dtype=torch.int32, device="cuda")
    sd = dict(BASE, steps=6, eta=1.0)
    with pytest.raises(drf.DrfError):
        den.sample(sd, I.CONSERVATIVE, 2, x, c)                       # needs a noise source
    a = den.sample_noise(sd, I.CONSERVATIVE, 2, x, c, seed=5)
    b = den.sample_noise(sd, I.CONSERVATIVE, 2, x, c, seed=5)
    assert torch.equal(a, b)                                          # reproducible
    assert not torch.equal(a, den.sample_noise(sd, I.CONSERVATIVE, 2, x, c, seed=6))
    # the generated stream and the same fields passed explicitly give the same result
    cnt = drf.noise_count(sd, I.CONSERVATIVE, 2)
    z = drf.normal_fill(5, 0, cnt, x.numel())
    assert torch.equal(a, den.sample_noise(sd, I.CONSERVATIVE, 2, x, c, z=z))
    # eta = 0 ignores the source; one step has no variance at all
    d0 = dict(BASE, steps=6)
    assert torch.equal(den.sample(d0, I.AGGRESSIVE, 3, x, c), den.sample_noise(d0, I.AGGRESSIVE, 3, x, c, seed=9))
    one = den.sample(dict(BASE, steps=1, eta=1.0), I.AGGRESSIVE, 3, x, c)
    assert torch.isfinite(one).all()
    # in place
    y = x.clone()
    den.sample_noise(sd, I.AGGRESSIVE, 2, y, c, seed=5, out=y)
    assert torch.equal(y, den.sample_noise(sd, I.AGGRESSIVE, 2, x, c, seed=5))
    den.close()
