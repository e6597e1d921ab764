"""Pins for the oracle's DiT forward, guidance and bf16 parameter rounding.

The paper treats the noise predictor as a black box, so nothing in it fixes the
DiT's values ("parity unpinned" by the paper).  The oracle's hand-written loops
are pinned here against an independent composition of torch float64 library
routines (linear, layer_norm, scaled_dot_product_attention, gelu, silu), against
structural invariants, and against special cases that collapse to a linear map."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_2603_25872_amd import inputs as I


def small_dit(cond, **kw):
    base = dict(depth=2, hidden=32, heads=4, mlp_ratio=4, patch=2, in_ch=4, lat_h=8, lat_w=6,
                dtype=I.F32, cond=cond, cond_dim={0: 12, 1: 10, 2: 20}[cond],
                ctx_len=5 if cond == I.COND_TEXT else 0)
    base.update(kw)
    return base


def make_cond(dit, slots, seed):
    rng = np.random.default_rng(seed)
    if dit["cond"] == I.COND_VECTOR:
        return rng.standard_normal((slots, dit["cond_dim"]))
    if dit["cond"] == I.COND_CLASS:
        return rng.integers(0, dit["cond_dim"] + 1, size=slots).astype(np.int32)
    return rng.standard_normal((slots, dit["ctx_len"], dit["cond_dim"]))


def torch_dit(dit, flat, x, t, cond, stop_blocks=-1):
    """The same network from torch float64 library routines."""
    W = {k: torch.from_numpy(np.array(v, np.float64)) for k, v in I.param_views(dit, flat).items()}
    D, h, p = dit["hidden"], dit["heads"], dit["patch"]
    x = torch.from_numpy(np.asarray(x, np.float64))
    S, C, H, Wd = x.shape
    gh, gw = H // p, Wd // p
    # patchify via unfold: channel-major, then dy, dx
    tok = F.unfold(x, kernel_size=p, stride=p).transpose(1, 2)          # [S, T, C*p*p]
    xs = F.linear(tok, W["patch_w"], W["patch_b"])
    q4 = D // 4
    om = torch.exp(-math.log(10000.0) * torch.arange(q4, dtype=torch.float64) / q4)
    py = torch.arange(gh, dtype=torch.float64).repeat_interleave(gw)
    px = torch.arange(gw, dtype=torch.float64).repeat(gh)
    pos = torch.cat([torch.sin(py[:, None] * om), torch.cos(py[:, None] * om),
                     torch.sin(px[:, None] * om), torch.cos(px[:, None] * om)], dim=1)
    xs = xs + pos
    tt = torch.from_numpy(np.asarray(t, np.float64))
    fr = torch.exp(-math.log(10000.0) * torch.arange(128, dtype=torch.float64) / 128)
    emb = torch.cat([torch.cos(tt[:, None] * fr), torch.sin(tt[:, None] * fr)], dim=1)
    c = F.linear(F.silu(F.linear(emb, W["t_w1"], W["t_b1"])), W["t_w2"], W["t_b2"])
    if dit["cond"] == I.COND_VECTOR:
        c = c + F.linear(torch.from_numpy(np.asarray(cond, np.float64)), W["c_w"], W["c_b"])
    elif dit["cond"] == I.COND_CLASS:
        c = c + W["table"][torch.from_numpy(np.asarray(cond)).long()]
    ca = F.silu(c)

    def heads(z):
        return z.reshape(z.shape[0], z.shape[1], h, D // h).transpose(1, 2)

    nblk = dit["depth"] if stop_blocks < 0 else stop_blocks
    for l in range(nblk):
        b = "blk%d." % l
        m = F.linear(ca, W[b + "ada_w"], W[b + "ada_b"]).chunk(6, dim=1)
        hcur = F.layer_norm(xs, (D,), eps=1e-6) * (1 + m[1][:, None]) + m[0][:, None]
        q, k, v = F.linear(hcur, W[b + "qkv_w"], W[b + "qkv_b"]).chunk(3, dim=2)
        a = F.scaled_dot_product_attention(heads(q), heads(k), heads(v)).transpose(1, 2).reshape(S, -1, D)
        xs = xs + m[2][:, None] * F.linear(a, W[b + "proj_w"], W[b + "proj_b"])
        if dit["cond"] == I.COND_TEXT:
            ctx = torch.from_numpy(np.asarray(cond, np.float64))
            q = F.linear(F.layer_norm(xs, (D,), eps=1e-6), W[b + "xq_w"], W[b + "xq_b"])
            k, v = F.linear(ctx, W[b + "xkv_w"], W[b + "xkv_b"]).chunk(2, dim=2)
            a = F.scaled_dot_product_attention(heads(q), heads(k), heads(v)).transpose(1, 2).reshape(S, -1, D)
            xs = xs + F.linear(a, W[b + "xo_w"], W[b + "xo_b"])
        hcur = F.layer_norm(xs, (D,), eps=1e-6) * (1 + m[4][:, None]) + m[3][:, None]
        mid = F.gelu(F.linear(hcur, W[b + "fc1_w"], W[b + "fc1_b"]), approximate="tanh")
        xs = xs + m[5][:, None] * F.linear(mid, W[b + "fc2_w"], W[b + "fc2_b"])
    if stop_blocks >= 0:
        return xs.numpy()
    m = F.linear(ca, W["fin_ada_w"], W["fin_ada_b"]).chunk(2, dim=1)
    hcur = F.layer_norm(xs, (D,), eps=1e-6) * (1 + m[1][:, None]) + m[0][:, None]
    out = F.linear(hcur, W["fin_w"], W["fin_b"])                        # [S, T, C*p*p]
    return F.fold(out.transpose(1, 2), (H, Wd), kernel_size=p, stride=p).numpy()


@pytest.mark.parametrize("cond", [I.COND_VECTOR, I.COND_CLASS, I.COND_TEXT])
@pytest.mark.parametrize("init", ["paper", "loud"])
def test_dit_matches_torch_float64(orc, cond, init):
    dit = small_dit(cond)
    assert orc.weight_count(dit) == I.param_count(dit)
    w = I.weights(dit, 11 + cond, init)
    rng = np.random.default_rng(20 + cond)
    slots = 3
    x = rng.standard_normal((slots, 4, dit["lat_h"], dit["lat_w"]))
    t = np.array([0, 517, 980], np.int32)
    cnd = make_cond(dit, slots, 30 + cond)
    got = orc.dit_eps(dit, w, x, t, cnd)
    want = torch_dit(dit, w, x, t, cnd)
    assert np.abs(want).max() > 1e-3
    np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-11)
    for k in range(dit["depth"] + 1):
        np.testing.assert_allclose(orc.dit_eps(dit, w, x, t, cnd, stop_blocks=k),
                                   torch_dit(dit, w, x, t, cnd, stop_blocks=k), rtol=1e-9, atol=1e-11)


def test_dit_head_dim_72_shape(orc):
    # hidden 144 / 2 heads = 72 per head, the DiT-XL head width
    dit = small_dit(I.COND_CLASS, hidden=144, heads=2, depth=1, lat_h=4, lat_w=4)
    w = I.weights(dit, 3, "loud")
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 4, 4, 4))
    t = np.array([40, 900], np.int32)
    cnd = np.array([10, 3], np.int32)
    np.testing.assert_allclose(orc.dit_eps(dit, w, x, t, cnd), torch_dit(dit, w, x, t, cnd),
                               rtol=1e-9, atol=1e-11)


def test_slots_are_independent_and_timestep_is_per_slot(orc):
    dit = small_dit(I.COND_CLASS)
    w = I.weights(dit, 1, "loud")
    rng = np.random.default_rng(6)
    x = rng.standard_normal((4, 4, dit["lat_h"], dit["lat_w"]))
    t = np.array([3, 400, 400, 999], np.int32)
    cnd = np.array([1, 2, 2, 10], np.int32)
    full = orc.dit_eps(dit, w, x, t, cnd)
    for j in range(4):
        one = orc.dit_eps(dit, w, x[j:j + 1], t[j:j + 1], cnd[j:j + 1])
        assert np.array_equal(one[0], full[j])
    # same x, different timestep -> different output
    two = orc.dit_eps(dit, w, np.stack([x[0], x[0]]), np.array([10, 900], np.int32), cnd[:2] * 0)
    assert np.abs(two[0] - two[1]).max() > 1e-3


def test_zero_gates_collapse_to_linear_map(orc):
    # With the adaLN projections of every block zeroed (gates = 0) the blocks are
    # identities and eps is patch-embed -> LayerNorm-modulate -> final Linear.
    dit = small_dit(I.COND_VECTOR)
    w = I.weights(dit, 2, "loud")
    v = I.param_views(dit, w)
    for l in range(dit["depth"]):
        v["blk%d.ada_w" % l][...] = 0
        v["blk%d.ada_b" % l][...] = 0
    rng = np.random.default_rng(7)
    x = rng.standard_normal((1, 4, dit["lat_h"], dit["lat_w"]))
    cnd = rng.standard_normal((1, dit["cond_dim"]))
    t = np.array([123], np.int32)
    got = orc.dit_eps(dit, w, x, t, cnd)
    dit0 = dict(dit, depth=0)
    keep = [n for n, _ in I.param_shapes(dit0)]
    w0 = np.concatenate([v[n].ravel() for n in keep])
    np.testing.assert_allclose(got, torch_dit(dit0, w0, x, t, cnd), rtol=1e-10, atol=1e-12)


def test_token_permutation_equivariance_without_position_code(orc):
    # Attention and per-token layers commute with a permutation of tokens.  Feed two
    # latents that differ by swapping two patches; outputs after removing the
    # position-dependent part must swap likewise.  Position code is additive, so
    # compare the DIFFERENCE between two inputs' residual streams at block 0.
    dit = small_dit(I.COND_CLASS, depth=0)
    w = I.weights(dit, 4, "loud")
    rng = np.random.default_rng(8)
    x = rng.standard_normal((1, 4, dit["lat_h"], dit["lat_w"]))
    xs = x.copy()
    # swap patch (0,0) with patch (1,2)
    xs[:, :, 0:2, 0:2], xs[:, :, 2:4, 4:6] = x[:, :, 2:4, 4:6], x[:, :, 0:2, 0:2]
    t = np.array([77], np.int32)
    c = np.array([0], np.int32)
    r0 = orc.dit_eps(dit, w, x, t, c, stop_blocks=0)[0]
    r1 = orc.dit_eps(dit, w, xs, t, c, stop_blocks=0)[0]
    gw = dit["lat_w"] // 2
    a, b = 0, 1 * gw + 2
    zero = orc.dit_eps(dit, w, np.zeros_like(x), t, c, stop_blocks=0)[0]   # bias + position code
    np.testing.assert_allclose(r1[a] - zero[a], r0[b] - zero[b], atol=1e-12)
    np.testing.assert_allclose(r1[b] - zero[b], r0[a] - zero[a], atol=1e-12)
    others = [i for i in range(r0.shape[0]) if i not in (a, b)]
    np.testing.assert_allclose(r1[others], r0[others], atol=1e-13)


# ------------------------------------------------------------------ guidance

def test_guidance_special_cases(orc):
    dit = small_dit(I.COND_CLASS)
    w = I.weights(dit, 5, "loud")
    rng = np.random.default_rng(9)
    x = rng.standard_normal((2, 4, dit["lat_h"], dit["lat_w"]))
    cnd = np.array([1, 7], np.int32)
    null = np.array([10, 10], np.int32)
    t = np.array([300, 300], np.int32)
    ec = orc.dit_eps(dit, w, x, t, cnd)
    eu = orc.dit_eps(dit, w, x, t, null)
    assert np.abs(ec - eu).max() > 1e-4
    np.testing.assert_allclose(orc.eps_guided(dit, w, x, 300, cnd, null, 1.0), ec, atol=1e-13)
    np.testing.assert_allclose(orc.eps_guided(dit, w, x, 300, cnd, null, 0.0), eu, atol=1e-13)
    np.testing.assert_allclose(orc.eps_guided(dit, w, x, 300, cnd, null, 4.0), eu + 4.0 * (ec - eu), atol=1e-12)
    np.testing.assert_allclose(orc.eps_guided(dit, w, x, 300, cnd, cnd, 4.0), ec, atol=1e-12)
    assert np.array_equal(orc.eps_guided(dit, w, x, 300, cnd, None, 4.0), ec)


# -------------------------------------------------------- bf16 parameter rounding

def test_bf16_rounding_is_rne_on_every_parameter(orc):
    dit = small_dit(I.COND_CLASS)
    w = I.weights(dit, 6, "loud")
    # plant exact ties and edge values among the parameters
    w[:6] = np.array([1.00390625, 1.01171875, -1.00390625, 3.0e-39, 65504.0, 0.0], np.float32)
    rng = np.random.default_rng(10)
    x = rng.standard_normal((1, 4, dit["lat_h"], dit["lat_w"]))
    t = np.array([42], np.int32)
    c = np.array([4], np.int32)
    got = orc.dit_eps(dict(dit, dtype=I.BF16), w, x, t, c)
    w_r = torch.from_numpy(w).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(w_r[:3], np.array([1.0, 1.015625, -1.0], np.float32))   # ties to even
    want = orc.dit_eps(dit, w_r, x, t, c)
    assert np.array_equal(got, want)
    assert np.abs(got - orc.dit_eps(dit, w, x, t, c)).max() > 0


def test_float_build_tracks_double_build(orc, orc32):
    dit = small_dit(I.COND_TEXT)
    w = I.weights(dit, 7, "loud")
    rng = np.random.default_rng(12)
    x = rng.standard_normal((2, 4, dit["lat_h"], dit["lat_w"]))
    t = np.array([5, 800], np.int32)
    cnd = make_cond(dit, 2, 13)
    a = orc.dit_eps(dit, w, x, t, cnd)
    b = orc32.dit_eps(dit, w, x, t, cnd)
    assert np.abs(a - b).max() / np.abs(a).max() < 2e-5


# ------------------------------------------------- whole path with the DiT inside

@pytest.mark.parametrize("mode", [I.CONSERVATIVE, I.AGGRESSIVE])
def test_sample_dit_equals_scheduler_with_guided_predictor(orc, mode):
    dit = small_dit(I.COND_CLASS, depth=1)
    w = I.weights(dit, 8, "loud")
    sd = dict(train_steps=1000, beta_start=1e-4, beta_end=0.02, steps=5)
    rng = np.random.default_rng(14)
    xT = rng.standard_normal((2, 4, dit["lat_h"], dit["lat_w"]))
    cnd = np.array([2, 9], np.int32)
    null = np.array([10, 10], np.int32)
    got = orc.sample_dit(dit, w, sd, mode, 2, xT, cnd, null, 3.0)

    def eps(x, s, tau):
        t = np.full(2, tau, np.int32)
        ec, eu = torch_dit(dit, w, x, t, cnd), torch_dit(dit, w, x, t, null)
        return eu + 3.0 * (ec - eu)

    want = orc.sample_with(sd, mode, 2, xT, eps)
    np.testing.assert_allclose(got, want, rtol=1e-8, atol=1e-10)
