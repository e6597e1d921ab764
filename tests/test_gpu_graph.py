"""drf_sample through a captured HIP graph against the same call launched kernel by kernel: every replay,
with the program's own eager work and synchronisations between the replays, must give the eager bits."""
import numpy as np
import pytest

from paper_2603_25872_amd import inputs as I

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
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


CASES = {
    "cfg1-f32": lambda: (I.config(1), {}),
    "cfg2-bf16-small": lambda: (I.config(2, depth=3, lat_h=16, lat_w=16), dict(steps=11)),
    "cfg3-bf16-guided": lambda: (I.config(3, depth=2, hidden=576, heads=8, lat_h=8, lat_w=8), dict(steps=9)),
    "text-bf16-guided": lambda: (I.config(4, depth=2, hidden=192, heads=3, lat_h=8, lat_w=8, cond_dim=64, ctx_len=9), dict(steps=7)),
    "cfg2-stochastic": lambda: (I.config(2, depth=2, lat_h=16, lat_w=16), dict(steps=8, eta=1.0)),
}


@pytest.mark.parametrize("case", sorted(CASES))
@pytest.mark.parametrize("first_mode", [1, 2])
def test_graph_replays_equal_the_eager_call(torch, drf, case, first_mode):
    cfg, so = CASES[case]()
    dit, sd = cfg["dit"], dict(cfg["sched"], **so)
    B = max(cfg["batch"], 2)
    den = drf.Denoiser(dit, I.weights(dit, 21, "loud"))
    xT = dev(torch, I.latent_noise(dit, B, 21))
    cond = dev(torch, I.conditioning(dit, B, 21))
    null = dev(torch, I.conditioning(dit, B, 21, null=True)) if cfg["guidance"] else None
    out = torch.empty_like(xT)
    stochastic = sd.get("eta", 0.0) != 0.0

    def call():
        if stochastic:
            return den.sample_noise(sd, cfg["mode"], cfg["n"], xT, cond, null, cfg["guidance"] or 0.0, seed=7, out=out)
        return den.sample(sd, cfg["mode"], cfg["n"], xT, cond, null, cfg["guidance"] or 0.0, out=out)

    den.use_graphs(0)
    want = call().clone()
    # a second input in the SAME buffers: a replay must read the live contents, not what it was captured with
    x2 = torch.randn_like(xT)
    keep = xT.clone()
    xT.copy_(x2)
    want2 = call().clone()
    xT.copy_(keep)
    assert not torch.equal(want, want2)

    den.use_graphs(first_mode)
    t = torch.randint(0, 1000, (3,), dtype=torch.int32, device="cuda")
    for it in range(6):                              # mode 1: eager, capture + replay, replays; mode 2: capture at once
        if it % 2 == 1:
            xT.copy_(x2)
        got = call()
        torch.cuda.synchronize()
        assert torch.equal(got, want2 if it % 2 == 1 else want), (case, it)
        xT.copy_(keep)
        # the program's own eager work between replays: another pass on the same handle, then a synchronisation
        den.eps_batched(xT[:1].repeat(3, 1, 1, 1), t, cond[:1].repeat(3, *([1] * (cond.dim() - 1))))
        torch.cuda.synchronize()
    st = den.graph_stats()
    assert st["failed"] == 0 and st["captured"] == 1 and st["replays"] == (5 if first_mode == 1 else 6), st
    # a pass that grows the workspace invalidates the captured graph: the next calls re-capture on the new buffers
    big = 4 * cfg["n"] * (2 if cfg["guidance"] else 1) * B
    den.eps_batched(xT[:1].repeat(big, 1, 1, 1), torch.zeros(big, dtype=torch.int32, device="cuda"),
                    cond[:1].repeat(big, *([1] * (cond.dim() - 1))))
    for it in range(3):
        assert torch.equal(call(), want), (case, "after growth", it)
    den.use_graphs(0)
    assert torch.equal(call(), want)
    den.close()


def test_graph_cache_keeps_several_argument_sets(torch, drf):
    """More argument sets than the handle keeps graphs for, cycled: every call still gives its eager result."""
    cfg = I.config(2, depth=2, lat_h=16, lat_w=16)
    dit = cfg["dit"]
    den = drf.Denoiser(dit, I.weights(dit, 22, "loud"))
    xT = dev(torch, I.latent_noise(dit, 2, 22))
    cond = dev(torch, I.conditioning(dit, 2, 22))
    sets = [(dict(cfg["sched"], steps=s), mode, n) for s in (5, 6, 7, 8) for mode in (0, 1) for n in (2, 3)][:11]
    den.use_graphs(0)
    want = [den.sample(sd, mode, n, xT, cond).clone() for sd, mode, n in sets]
    den.use_graphs(1)
    outs = [torch.empty_like(xT) for _ in sets]
    for rep in range(4):
        for i, (sd, mode, n) in enumerate(sets):
            den.sample(sd, mode, n, xT, cond, out=outs[i])
        torch.cuda.synchronize()
        for i in range(len(sets)):
            assert torch.equal(outs[i], want[i]), (rep, i)
    st = den.graph_stats()
    assert st["failed"] == 0 and st["captured"] <= 8, st
    den.close()
