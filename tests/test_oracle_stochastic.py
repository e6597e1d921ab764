"""Pins for the oracle's stochastic DDIM skip (sigma > 0), the DDPM skip transition, the
Euler skip, the noise-consuming schedulers and the counter-based normal stream.

Every expected value here comes from outside the oracle: the textbook one-step DDPM
posterior, a brute-force product of Gaussians on a grid, closed forms, published Philox
test vectors, or a block written out by hand with explicit noise fields.  No GPU."""
import math

import numpy as np
import pytest
from scipy import stats

from paper_2603_25872_amd import inputs as I

BASE = dict(train_steps=1000, beta_start=1e-4, beta_end=0.02, steps=20)
CONS, AGGR = I.CONSERVATIVE, I.AGGRESSIVE
DDIM, DDPM, EULER = 0, 1, 2


def sched(S, **kw):
    return dict(BASE, steps=S, **kw)


def nonlinear_eps(x, s, tau):
    return np.tanh(1.3 * x) * math.cos(0.01 * tau + 0.2) + 0.1 * np.sin(x * (1 + 0.003 * tau))


# ------------------------------------------------- posterior variance and mean

def test_posterior_var_k1_is_textbook_ddpm(orc):
    # Eq. ddpm_skip_reverse_detail at k = 1 must be the usual DDPM posterior variance
    # beta~_t = (1 - abar_{t-1}) / (1 - abar_t) * beta_t  (Ho et al., Eq. 7).
    betas = np.linspace(1e-4, 0.02, 1000)
    ab = np.cumprod(1 - betas)
    for t in (1, 2, 17, 500, 999):
        want = (1 - ab[t - 1]) / (1 - ab[t]) * betas[t]
        assert abs(orc.posterior_var(ab[t], ab[t - 1]) / want - 1) < 1e-12


def test_ddpm_mean_k1_is_textbook_ddpm(orc):
    # k = 1 mean in the epsilon parameterisation: (x - beta_t / sqrt(1 - abar_t) eps) / sqrt(1 - beta_t).
    betas = np.linspace(1e-4, 0.02, 1000)
    ab = np.cumprod(1 - betas)
    rng = np.random.default_rng(11)
    x, eps = rng.standard_normal(50), rng.standard_normal(50)
    for t in (1, 40, 700, 999):
        want = (x - betas[t] / math.sqrt(1 - ab[t]) * eps) / math.sqrt(1 - betas[t])
        np.testing.assert_allclose(orc.ddpm_skip(x, eps, None, ab[t], ab[t - 1]), want, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("a_from,a_to", [(0.3, 0.8), (0.05, 0.2), (0.6, 0.95), (0.2, 0.25)])
def test_ddpm_skip_is_bayes_product_brute_force(orc, a_from, a_to):
    # Eq. ddpm_bayes for scalars: q(x_to | x_from, x0) ~ q(x_from | x_to) q(x_to | x0), with
    # q(x_from | x_to) = N(sqrt(a_from/a_to) x_to, 1 - a_from/a_to) (forward chain composed),
    # q(x_to | x0) = N(sqrt(a_to) x0, 1 - a_to).  Moments by quadrature on a fine grid.
    x0, x_from = 0.83, -0.41
    r = a_from / a_to
    grid = np.linspace(-12, 12, 400001)
    logp = -(x_from - math.sqrt(r) * grid) ** 2 / (2 * (1 - r)) - (grid - math.sqrt(a_to) * x0) ** 2 / (2 * (1 - a_to))
    p = np.exp(logp - logp.max())
    p /= p.sum()
    mean = float((p * grid).sum())
    var = float((p * (grid - mean) ** 2).sum())
    # the oracle takes (x, eps): pick eps so that the predicted x0 is the one above
    eps = (x_from - math.sqrt(a_from) * x0) / math.sqrt(1 - a_from)
    got = orc.ddpm_skip(np.array([x_from]), np.array([eps]), None, a_from, a_to)[0]
    assert abs(got - mean) < 1e-8
    assert abs(orc.posterior_var(a_from, a_to) - var) < 1e-8
    # the noise enters with the posterior standard deviation
    got1 = orc.ddpm_skip(np.array([x_from]), np.array([eps]), np.array([1.0]), a_from, a_to)[0]
    assert abs((got1 - got) - math.sqrt(var)) < 1e-8


def test_ddpm_skip_to_clean_data_returns_predicted_x0(orc):
    rng = np.random.default_rng(12)
    x, eps, z = rng.standard_normal(9), rng.standard_normal(9), rng.standard_normal(9)
    a = 0.37
    want = (x - math.sqrt(1 - a) * eps) / math.sqrt(a)
    np.testing.assert_allclose(orc.ddpm_skip(x, eps, z, a, 1.0), want, atol=1e-13)
    assert orc.posterior_var(a, 1.0) == 0.0


# ------------------------------------------------------- stochastic DDIM skip

@pytest.mark.parametrize("a_from,a_to", [(0.3, 0.8), (1.06e-4, 0.5), (0.7, 0.71), (0.2, 1.0)])
def test_ddim_eta1_equals_ddpm_posterior(orc, a_from, a_to):
    # The DDIM skip with the DDPM-induced variance is the DDPM skip: same mean, same noise scale.
    rng = np.random.default_rng(13)
    x, eps, z = rng.standard_normal(40), rng.standard_normal(40), rng.standard_normal(40)
    sg = orc.sigma(1.0, a_from, a_to)
    np.testing.assert_allclose(orc.skip_eta(x, eps, z, a_from, a_to, sg), orc.ddpm_skip(x, eps, z, a_from, a_to),
                               rtol=1e-11, atol=1e-11)


def test_sigma_scales_with_eta(orc):
    a_from, a_to = 0.2, 0.6
    sd1 = orc.sigma(1.0, a_from, a_to)
    assert abs(sd1 ** 2 - (1 - a_from / a_to) * (1 - a_to) / (1 - a_from)) < 1e-15
    assert abs(orc.sigma(0.35, a_from, a_to) - 0.35 * sd1) < 1e-15
    assert orc.sigma(0.0, a_from, a_to) == 0.0


@pytest.mark.parametrize("eta", [0.0, 0.3, 1.0])
def test_skip_eta_keeps_the_marginal(orc, eta):
    # Eq. ddim_consistency: from x_t on the marginal with the true noise, the skip gives
    # sqrt(a_to) x0 + sqrt(1 - a_to - sigma^2) eps + sigma z, whose noise part has total
    # variance 1 - a_to.  Unit vectors separate the three coefficients.
    a_from, a_to = 0.15, 0.55
    sg = orc.sigma(eta, a_from, a_to)
    x0 = np.array([1.0, 0.0, 0.0])
    eps = np.array([0.0, 1.0, 0.0])
    z = np.array([0.0, 0.0, 1.0])
    xt = math.sqrt(a_from) * x0 + math.sqrt(1 - a_from) * eps
    out = orc.skip_eta(xt, eps, z, a_from, a_to, sg)
    assert abs(out[0] - math.sqrt(a_to)) < 1e-14
    assert abs(out[2] - sg) < 1e-15
    assert abs(out[1] ** 2 + out[2] ** 2 - (1 - a_to)) < 1e-14
    assert out[1] > 0


def test_skip_eta_zero_sigma_is_the_deterministic_skip(orc):
    rng = np.random.default_rng(14)
    x, eps, z = rng.standard_normal(33), rng.standard_normal(33), rng.standard_normal(33)
    assert np.array_equal(orc.skip_eta(x, eps, z, 0.2, 0.7, 0.0), orc.skip(x, eps, 0.2, 0.7))
    assert np.array_equal(orc.skip_eta(x, eps, None, 0.2, 0.7, 0.0), orc.skip(x, eps, 0.2, 0.7))


def test_more_fresh_noise_keeps_less_of_the_old_noise(orc):
    # the coefficient on eps shrinks as sigma grows, and the total stays on the marginal
    a_from, a_to = 0.1, 0.45
    x, eps = np.zeros(1), np.ones(1)
    base = -math.sqrt(a_to) * math.sqrt(1 - a_from) / math.sqrt(a_from)     # from the predicted x0
    dirs = [orc.skip_eta(x, eps, None, a_from, a_to, orc.sigma(eta, a_from, a_to))[0] - base for eta in (0.0, 0.5, 1.0)]
    assert dirs[0] > dirs[1] > dirs[2] > 0
    for eta, d in zip((0.0, 0.5, 1.0), dirs):
        assert abs(d * d + orc.sigma(eta, a_from, a_to) ** 2 - (1 - a_to)) < 1e-13


# ----------------------------------------------------------------- Euler skip

def test_euler_skip_closed_forms(orc):
    rng = np.random.default_rng(15)
    x, v = rng.standard_normal(21), rng.standard_normal(21)
    np.testing.assert_allclose(orc.euler_skip(x, v, 0.9, 0.4), x - 0.5 * v, atol=1e-15)
    assert np.array_equal(orc.euler_skip(x, v, 0.3, 0.3), x)
    # constant velocity: two steps compose into one
    two = orc.euler_skip(orc.euler_skip(x, v, 1.0, 0.6), v, 0.6, 0.1)
    np.testing.assert_allclose(two, orc.euler_skip(x, v, 1.0, 0.1), atol=1e-15)
    # straight-line flow x_sigma = (1 - sigma) x0 + sigma e with its true velocity e - x0:
    # any skip lands exactly on the line, a skip to 0 returns x0
    x0, e = rng.standard_normal(21), rng.standard_normal(21)
    xs = 0.3 * x0 + 0.7 * e
    np.testing.assert_allclose(orc.euler_skip(xs, e - x0, 0.7, 0.0), x0, atol=1e-15)
    np.testing.assert_allclose(orc.euler_skip(xs, e - x0, 0.7, 0.25), 0.75 * x0 + 0.25 * e, atol=1e-15)


def test_sigma_grid_and_network_time(orc):
    sd = sched(50, sampler=EULER)
    assert orc.sigma_at(sd, 0) == 0.0 and orc.sigma_at(sd, 50) == 1.0
    assert abs(orc.sigma_at(sd, 17) - 17 / 50) < 1e-16
    assert [orc.net_time(sd, s) for s in (1, 2, 50)] == [20, 40, 1000]
    sh = sched(50, sampler=EULER, shift=3.0)
    assert orc.sigma_at(sh, 0) == 0.0 and abs(orc.sigma_at(sh, 50) - 1.0) < 1e-16
    assert abs(orc.sigma_at(sh, 25) - 0.75) < 1e-15          # 3 * 0.5 / (1 + 2 * 0.5)
    assert orc.net_time(sh, 25) == 750
    grid = [orc.sigma_at(sh, s) for s in range(51)]
    assert all(b > a for a, b in zip(grid, grid[1:]))
    # the DDIM samplers keep the strided timestep map
    assert orc.net_time(sched(50), 50) == 980 and orc.net_time(sched(50, sampler=DDPM), 1) == 0


# ---------------------------------------------------------------- schedulers

@pytest.mark.parametrize("mode", [CONS, AGGR])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 7])
@pytest.mark.parametrize("S", [1, 2, 5, 20])
def test_noise_count_is_drafts_plus_updates(orc, mode, n, S):
    sd = sched(S, eta=1.0)
    rows = orc.plan(sd, mode, n)
    assert orc.noise_count(sd, mode, n) == int((rows[:, 1] != 0).sum())
    # every sampling step is one transition into the kept trajectory; the other draws are drafts
    kept = int((rows[:, 1] == 2).sum()) + len({int(r[2]) for r in rows if r[1] == 1})
    assert kept == S


def seq_stochastic(sd, xT, eps_fn, z, sampler, eta):
    """Sequential ancestral sampling, textbook form, noise field i used by step i."""
    ab = np.cumprod(1.0 - np.linspace(sd["beta_start"], sd["beta_end"], sd["train_steps"]))
    stride = sd["train_steps"] // sd["steps"]
    a = lambda s: 1.0 if s == 0 else ab[(s - 1) * stride]
    x = np.array(xT, np.float64)
    for i, s in enumerate(range(sd["steps"], 0, -1)):
        e = eps_fn(x, s, (s - 1) * stride)
        af, at = a(s), a(s - 1)
        var = (1 - af / at) * (1 - at) / (1 - af)
        x0 = (x - math.sqrt(1 - af) * e) / math.sqrt(af)
        if sampler == DDPM:
            x = (math.sqrt(af / at) * (1 - at) * x + math.sqrt(at) * (1 - af / at) * x0) / (1 - af) + math.sqrt(var) * z[i]
        else:
            sg = eta * math.sqrt(var)
            x = math.sqrt(at) * x0 + math.sqrt(1 - at - sg * sg) * e + sg * z[i]
    return x


@pytest.mark.parametrize("mode", [CONS, AGGR])
@pytest.mark.parametrize("S", [1, 2, 7, 20])
@pytest.mark.parametrize("sampler,eta", [(DDIM, 0.4), (DDIM, 1.0), (DDPM, 0.0)])
def test_n1_is_sequential_stochastic_sampling(orc, mode, S, sampler, eta):
    # block size 1: each step is one draft (aggressive) or one update (conservative) and draws one field
    sd = sched(S, eta=eta, sampler=sampler)
    rng = np.random.default_rng(16)
    xT = rng.standard_normal((2, 3, 5))
    cnt = orc.noise_count(sd, mode, 1)
    z = rng.standard_normal((cnt,) + xT.shape)
    got = orc.sample_with(sd, mode, 1, xT, nonlinear_eps, z=z)
    if mode == AGGR:
        zs = z                       # one draft per step, no refine draws
        assert cnt == S
    else:
        # conservative n = 1: anchor s drafts s-1 (one draw) and refines to s-2 (one draw); a lone last step draws one
        zs = z
        assert cnt == S
    np.testing.assert_allclose(got, seq_stochastic(sd, xT, nonlinear_eps, zs, sampler, eta), rtol=1e-9, atol=1e-9)


def _step(orc, sd, x, e, z, a, b, eta):
    af, at = orc.abar_at(sd, a), orc.abar_at(sd, b)
    sg = eta * math.sqrt((1 - af / at) * (1 - at) / (1 - af))
    A = math.sqrt(at / af)
    return A * x + (math.sqrt(1 - at - sg * sg) - A * math.sqrt(1 - af)) * e + sg * z


def test_aggressive_block_by_hand_with_noise(orc):
    # Algorithm 1, S = 5, k = 2, eta = 0.7: draws in order z0 (draft 5->4), z1 (draft 5->3), z2 (refine 4->3),
    # z3 (draft 3->2), z4 (draft 3->1), z5 (refine 2->1), z6 (draft 1->0).
    eta = 0.7
    sd = sched(5, eta=eta)
    f = nonlinear_eps
    tau = lambda s: orc.tau(sd, s)
    rng = np.random.default_rng(17)
    x5 = rng.standard_normal((2, 6))
    z = rng.standard_normal((7, 2, 6))
    assert orc.noise_count(sd, AGGR, 2) == 7
    st = lambda x, e, zz, a, b: _step(orc, sd, x, e, zz, a, b, eta)
    e5 = f(x5, 5, tau(5))
    d4, d3 = st(x5, e5, z[0], 5, 4), st(x5, e5, z[1], 5, 3)
    e4, e3 = f(d4, 4, tau(4)), f(d3, 3, tau(3))
    x3 = st(d4, e4, z[2], 4, 3)
    d2, d1 = st(x3, e3, z[3], 3, 2), st(x3, e3, z[4], 3, 1)
    e2, e1 = f(d2, 2, tau(2)), f(d1, 1, tau(1))
    x1 = st(d2, e2, z[5], 2, 1)
    x0 = st(x1, e1, z[6], 1, 0)
    got = orc.sample_with(sd, AGGR, 2, x5, f, z=z)
    np.testing.assert_allclose(got, x0, atol=1e-12)
    # the draws matter, and their order matters
    assert np.abs(got - orc.sample_with(sd, AGGR, 2, x5, f, z=z[::-1])).max() > 1e-3
    assert np.abs(got - orc.sample_with(sd, AGGR, 2, x5, f, z=None)).max() > 1e-3


def test_conservative_block_by_hand_with_noise(orc):
    # Algorithm 2, S = 4, k = 2, eta = 1: solo 4; drafts 4->3 (z0), 4->2 (z1); refine 3->2 (z2), 2->1 (z3);
    # solo 1; last step 1->0 (z4, sigma = 0).
    eta = 1.0
    sd = sched(4, eta=eta)
    f = nonlinear_eps
    tau = lambda s: orc.tau(sd, s)
    rng = np.random.default_rng(18)
    x4 = rng.standard_normal((1, 7))
    z = rng.standard_normal((5, 1, 7))
    assert orc.noise_count(sd, CONS, 2) == 5
    st = lambda x, e, zz, a, b: _step(orc, sd, x, e, zz, a, b, eta)
    e4 = f(x4, 4, tau(4))
    d3, d2 = st(x4, e4, z[0], 4, 3), st(x4, e4, z[1], 4, 2)
    e3, e2 = f(d3, 3, tau(3)), f(d2, 2, tau(2))
    x2 = st(d3, e3, z[2], 3, 2)
    x1 = st(x2, e2, z[3], 2, 1)
    x0 = st(x1, f(x1, 1, tau(1)), z[4], 1, 0)
    np.testing.assert_allclose(orc.sample_with(sd, CONS, 2, x4, f, z=z), x0, atol=1e-12)
    # the transition onto clean data has no variance: its field is drawn but has no effect
    z2 = z.copy()
    z2[4] += 5.0
    np.testing.assert_allclose(orc.sample_with(sd, CONS, 2, x4, f, z=z2), x0, atol=1e-12)


@pytest.mark.parametrize("mode", [CONS, AGGR])
@pytest.mark.parametrize("n", [2, 3, 5])
def test_ddpm_sampler_equals_ddim_eta1_sampler(orc, mode, n):
    rng = np.random.default_rng(19)
    xT = rng.standard_normal((2, 10))
    sd1, sdp = sched(11, eta=1.0), sched(11, sampler=DDPM)
    z = rng.standard_normal((orc.noise_count(sd1, mode, n), 2, 10))
    assert orc.noise_count(sdp, mode, n) == z.shape[0]
    np.testing.assert_allclose(orc.sample_with(sdp, mode, n, xT, nonlinear_eps, z=z),
                               orc.sample_with(sd1, mode, n, xT, nonlinear_eps, z=z), rtol=1e-9, atol=1e-9)


@pytest.mark.parametrize("mode", [CONS, AGGR])
@pytest.mark.parametrize("n", [1, 2, 3, 8])
@pytest.mark.parametrize("shift", [1.0, 3.0])
def test_euler_constant_velocity_telescopes(orc, mode, n, shift):
    # constant v: every path through drafts and refinements sums to (sigma_0 - sigma_S) v = -v
    sd = sched(10, sampler=EULER, shift=shift)
    rng = np.random.default_rng(21)
    xT, c = rng.standard_normal((2, 6)), rng.standard_normal((2, 6))
    got = orc.sample_with(sd, mode, n, xT, lambda x, s, t: c)
    np.testing.assert_allclose(got, xT - c, atol=1e-13)


@pytest.mark.parametrize("mode", [CONS, AGGR])
@pytest.mark.parametrize("shift", [1.0, 2.5])
def test_euler_n1_is_plain_euler(orc, mode, shift):
    S = 9
    sd = sched(S, sampler=EULER, shift=shift)
    sig = lambda s: shift * (s / S) / (1 + (shift - 1) * (s / S))
    f = lambda x, s, t: np.sin(2 * x) + 0.001 * t
    xT = np.random.default_rng(22).standard_normal((1, 13))
    x = xT.copy()
    for s in range(S, 0, -1):
        x = x + (sig(s - 1) - sig(s)) * f(x, s, int(math.floor(sig(s) * 1000 + 0.5)))
    np.testing.assert_allclose(orc.sample_with(sd, mode, 1, xT, f), x, atol=1e-12)


def test_euler_linear_field_block_closed_form(orc):
    # v = a x: a conservative block S = 3, k = 2 is a product of scalar factors:
    #   d2 = (1 + h32 a) x3, d1 = (1 + h31 a) x3, x1 = (1 + h21 a) d2, x0 = x1 + h10 a d1.
    a = 0.8
    sd = sched(3, sampler=EULER)
    h = lambda f, t: (t - f) / 3.0
    x3 = np.array([[1.5, -2.0]])
    d2, d1 = (1 + h(3, 2) * a) * x3, (1 + h(3, 1) * a) * x3
    x1 = (1 + h(2, 1) * a) * d2
    x0 = x1 + h(1, 0) * a * d1
    np.testing.assert_allclose(orc.sample_with(sd, CONS, 2, x3, lambda x, s, t: a * x), x0, atol=1e-14)


def test_unknown_sampler_rejected(orc):
    with pytest.raises(ValueError):
        orc.plan(sched(5, sampler=3), CONS, 2)


# ------------------------------------------------------------- noise stream

def test_philox_known_answers(orc):
    # Test vectors of Philox4x32-10 distributed with the Random123 library (Salmon et al., SC'11).
    assert orc.philox([0, 0, 0, 0], [0, 0]) == [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]
    assert orc.philox([0xffffffff] * 4, [0xffffffff] * 2) == [0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd]
    assert orc.philox([0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], [0xa4093822, 0x299f31d0]) == \
        [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1]


def test_normal_fill_is_standard_normal(orc):
    z = orc.normal_fill(1234567, 0, 4, 250000).ravel()
    assert abs(z.mean()) < 4e-3 and abs(z.var() - 1) < 6e-3
    assert abs(stats.skew(z)) < 1e-2 and abs(stats.kurtosis(z)) < 2e-2
    assert stats.kstest(z[:200000], "norm").pvalue > 1e-3
    # neighbours (the cos / sin pair, the two pairs of a block, consecutive blocks) are uncorrelated
    for lag in (1, 2, 3, 4, 5):
        assert abs(np.corrcoef(z[:-lag], z[lag:])[0, 1]) < 5e-3


def test_normal_fill_layout(orc):
    # field f, element e depends only on (seed, f, e): ragged tails, field offsets and seeds
    a = orc.normal_fill(99, 0, 3, 1003)
    assert np.array_equal(orc.normal_fill(99, 1, 2, 1003), a[1:])
    assert np.array_equal(orc.normal_fill(99, 0, 3, 17)[:, :17], a[:, :17])
    assert np.abs(orc.normal_fill(100, 0, 1, 1003) - a[0]).max() > 0.5
    assert len(np.unique(a)) == a.size
    # element 4q+j comes from block q word pair: Box-Muller written out
    r = orc.philox([5, 0, 2, 0], [99, 0])
    u = [((w >> 9) + 0.5) / 2 ** 23 for w in r]
    want = [math.sqrt(-2 * math.log(u[0])) * math.cos(2 * math.pi * u[1]),
            math.sqrt(-2 * math.log(u[0])) * math.sin(2 * math.pi * u[1]),
            math.sqrt(-2 * math.log(u[2])) * math.cos(2 * math.pi * u[3]),
            math.sqrt(-2 * math.log(u[2])) * math.sin(2 * math.pi * u[3])]
    np.testing.assert_allclose(a[2, 20:24], want, rtol=1e-12)
    # the seed's high word is the second key word
    b = orc.normal_fill((7 << 32) | 99, 0, 1, 8)
    r = orc.philox([0, 0, 0, 0], [99, 7])
    u0, u1 = ((r[0] >> 9) + 0.5) / 2 ** 23, ((r[1] >> 9) + 0.5) / 2 ** 23
    assert abs(b[0, 0] - math.sqrt(-2 * math.log(u0)) * math.cos(2 * math.pi * u1)) < 1e-12


def test_float_build_of_the_stochastic_path_tracks_double(orc, orc32):
    sd = sched(10, eta=1.0)
    rng = np.random.default_rng(23)
    xT = rng.standard_normal((2, 12))
    z = rng.standard_normal((orc.noise_count(sd, CONS, 3), 2, 12))
    a = orc.sample_with(sd, CONS, 3, xT, nonlinear_eps, z=z)
    b = orc32.sample_with(sd, CONS, 3, xT, nonlinear_eps, z=z)
    assert np.abs(a - b).max() < 5e-5 * max(1.0, np.abs(a).max())
