"""Kernel-level parity through the measurement hooks: every tile shape of the bf16 GEMM and
the bf16 attention kernel against the oracle's plain loops, at shapes that leave ragged
tiles in every dimension, and the DiT-XL-shaped pass at its benchmark launch size on
sampled slots."""
import numpy as np
import pytest

from paper_2603_25872_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available()
    return t


@pytest.fixture(scope="module")
def drf():
    from paper_2603_25872_amd import drf as d
    d.lib()
    return d


def bf16_round(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch.bfloat16)


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("M,N,K", [(300, 292, 128), (517, 1156, 192), (1024, 576, 64), (33, 8, 64), (260, 148, 384)])
def test_gemm_bf16_every_tile_shape(torch, drf, orc, variant, M, N, K):
    rng = np.random.default_rng(M + N + K)
    A = bf16_round(torch, rng.standard_normal((M, K)))
    W = bf16_round(torch, rng.standard_normal((N, K)) * 0.1)
    b = rng.standard_normal(N).astype(np.float32)
    if variant == 8 and K % 128:                 # the split-K tile takes two 64-wide k-tiles per step
        with pytest.raises(drf.DrfError):
            drf.probe_gemm_bf16(A.cuda(), W.cuda(), torch.from_numpy(b).cuda(), variant=variant)
        return
    out = drf.probe_gemm_bf16(A.cuda(), W.cuda(), torch.from_numpy(b).cuda(), variant=variant).float().cpu().numpy()
    want = orc.linear(A.float().numpy(), W.float().numpy(), b)
    err = np.abs(out - want).max() / np.abs(want).max()
    assert err < 6e-3, err                       # bf16 rounding of the stored result: 2^-8 relative at worst


@pytest.mark.parametrize("M,N,K", [(512, 1152, 4608), (300, 292, 2304), (1024, 576, 2304), (130, 132, 2560)])
def test_gemm_bf16_split_k(torch, drf, orc, M, N, K):
    """Few 128 x 128 tiles and a long K: K is split across workgroups and the partial tiles are added by a second
    launch (5 or 6 splits here); same tolerance as the unsplit tile, whose result it must also track closely."""
    rng = np.random.default_rng(M + N + K)
    A = bf16_round(torch, rng.standard_normal((M, K)))
    W = bf16_round(torch, rng.standard_normal((N, K)) * 0.1)
    b = rng.standard_normal(N).astype(np.float32)
    out = drf.probe_gemm_bf16(A.cuda(), W.cuda(), torch.from_numpy(b).cuda(), variant=10).float().cpu().numpy()
    again = drf.probe_gemm_bf16(A.cuda(), W.cuda(), torch.from_numpy(b).cuda(), variant=10).float().cpu().numpy()
    assert np.array_equal(out, again)            # fixed summation order
    whole = drf.probe_gemm_bf16(A.cuda(), W.cuda(), torch.from_numpy(b).cuda(), variant=5).float().cpu().numpy()
    want = orc.linear(A.float().numpy(), W.float().numpy(), b)
    scale = np.abs(want).max()
    assert np.abs(out - want).max() / scale < 6e-3
    assert np.abs(out - whole).max() / scale < 6e-3   # both are bf16 roundings of nearly the same fp32 sums


def test_gemm_bf16_rejects_bad_k(torch, drf):
    A = torch.zeros((64, 72), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((64, 72), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(drf.DrfError):
        drf.probe_gemm_bf16(A, W, torch.zeros(64, device="cuda"))


@pytest.mark.parametrize("slots,T,H,d", [(3, 256, 2, 72), (2, 77, 3, 64), (5, 15, 4, 32), (1, 300, 1, 96), (2, 130, 2, 48),
                                          (1, 1, 2, 16), (2, 192, 1, 80), (1, 129, 1, 80), (2, 640, 2, 72), (1, 255, 2, 24),
                                          (40, 200, 8, 72), (65, 136, 4, 40)])     # more work items than CUs
def test_attention_bf16_shapes(torch, drf, orc, slots, T, H, d):
    rng = np.random.default_rng(T + d)
    qkv = bf16_round(torch, rng.standard_normal((slots * T, 3 * H * d)) * 1.5)
    out = drf.probe_attn_bf16(qkv.cuda(), slots, T, H, d).float().cpu().numpy()
    want = orc.attention_packed(qkv.float().numpy(), T, H, d)
    err = np.abs(out - want).max() / np.abs(want).max()
    assert err < 1.5e-2, err


def test_attention_bf16_large_scores_and_lazy_rescale(torch, drf, orc):
    # score ranges far beyond the lazy-rescale headroom, increasing along kv so the reference moves often
    slots, T, H, d = 1, 512, 1, 64
    rng = np.random.default_rng(3)
    q = rng.standard_normal((T, d)) * 4
    k = rng.standard_normal((T, d)) * np.linspace(0.2, 6, T)[:, None]
    v = rng.standard_normal((T, d))
    qkv = bf16_round(torch, np.concatenate([q, k, v], axis=1))
    out = drf.probe_attn_bf16(qkv.cuda(), slots, T, H, d).float().cpu().numpy()
    want = orc.attention_packed(qkv.float().numpy(), T, H, d)
    assert np.isfinite(out).all()
    assert np.abs(out - want).max() / np.abs(want).max() < 2e-2


def test_config3_pass_at_benchmark_size_sampled_slots(torch, drf, orc):
    """The 64-slot draft pass of configuration 3 (8 drafts-by-guidance groups of batch 8, distinct
    timesteps per group) as bench.py launches it; the oracle evaluates two sampled slots."""
    cfg = I.config(3)
    dit = cfg["dit"]
    w = I.weights(dit, 3)
    den = drf.Denoiser(dit, w)
    slots = cfg["n"] * 2 * cfg["batch"]
    rng = np.random.default_rng(33)
    x = rng.standard_normal((slots, 4, 32, 32)).astype(np.float32)
    stride = 1000 // cfg["sched"]["steps"]
    t = np.repeat(np.array([(49 - i) * stride for i in range(4)], np.int32), 16)       # tau of s = 50..47, per group
    cls = I.conditioning(dit, slots, 3)
    cls[1::2] = dit["cond_dim"]                                                         # null class on odd slots
    got = den.eps_batched(torch.from_numpy(x).cuda(), torch.from_numpy(t).cuda(), torch.from_numpy(cls).cuda())
    got = got.cpu().numpy()
    den.close()
    assert np.isfinite(got).all()
    wd = orc.prepare_weights(w)
    for j in (5, 62):
        want = orc.dit_eps(dit, wd, x[j:j + 1], t[j:j + 1], cls[j:j + 1])[0]
        err = np.abs(got[j] - want).max() / np.abs(want).max()
        assert err < 2e-2, (j, err)


@pytest.mark.parametrize("g,n_chain,n_draft", [(2, 4, 4), (1, 3, 0), (2, 0, 4), (1, 1, 1)])
def test_fused_update_probe_equals_its_parts(torch, drf, orc, g, n_chain, n_draft):
    """The measurement hook that launches the fused guidance + chain + draft update once, against the same steps
    made of refine_step / skip_transition calls and against the oracle's operator."""
    sd = dict(train_steps=1000, beta_start=1e-4, beta_end=0.02, steps=50, eta=0.0)
    rng = np.random.default_rng(g * 100 + n_chain * 10 + n_draft)
    shape, s_from, w = (3, 4, 8, 8), 20, 4.0
    x = rng.standard_normal(shape).astype(np.float32)
    eps = rng.standard_normal((max(n_chain, 1), g) + shape).astype(np.float32)
    xd, ed = torch.from_numpy(x).cuda(), torch.from_numpy(eps).cuda()
    x_out, drafts = drf.probe_update_fused(sd, s_from, n_chain, n_draft, g, w, xd, ed)
    guided = ed[:, 0] if g == 1 else ed[:, 1] + w * (ed[:, 0] - ed[:, 1])
    y, s = xd, s_from
    want = x.astype(np.float64)
    gn = guided.cpu().numpy().astype(np.float64)
    for i in range(n_chain):
        y = drf.refine_step(sd, y, guided[i].contiguous(), s)
        want = orc.skip(want, gn[i], orc.abar_at(sd, s), orc.abar_at(sd, s - 1))
        s -= 1
    assert np.abs(x_out.cpu().numpy() - y.cpu().numpy()).max() < 1e-5
    assert np.abs(x_out.cpu().numpy() - want).max() / np.abs(want).max() < 1e-5
    if n_draft:
        anchor = guided[n_chain - 1 if n_chain else 0].contiguous()
        parts = drf.skip_transition(sd, y, anchor, s, [s - j - 1 for j in range(n_draft)])
        assert np.abs(drafts.cpu().numpy() - parts.cpu().numpy()).max() < 1e-5
