"""The entry point that allocates nothing, drf_eps_batched_static, against drf_eps_batched: same kernels on
the library's static scratch array instead of the handle's workspace, so the results are the same bits.
Two calls in a row, the second with a smaller input (the array keeps the first call's contents)."""
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


def make(torch, dit, slots, seed):
    rng = np.random.default_rng(seed)
    x = torch.from_numpy(rng.standard_normal((slots, dit["in_ch"], dit["lat_h"], dit["lat_w"])).astype(np.float32)).cuda()
    t = torch.from_numpy(rng.integers(0, 1000, slots).astype(np.int32)).cuda()
    if dit["cond"] == I.COND_CLASS:
        c = torch.from_numpy(rng.integers(0, dit["cond_dim"] + 1, slots).astype(np.int32)).cuda()
    elif dit["cond"] == I.COND_VECTOR:
        c = torch.from_numpy(rng.standard_normal((slots, dit["cond_dim"])).astype(np.float32)).cuda()
    else:
        c = torch.from_numpy(rng.standard_normal((slots, dit["ctx_len"], dit["cond_dim"])).astype(np.float32)).cuda()
    return x, t, c


@pytest.mark.parametrize("which", ["cfg1-f32", "cfg2-bf16", "text-bf16"])
def test_static_scratch_entry_matches_the_allocating_one(torch, drf, which):
    if which == "cfg1-f32":
        dit, first, second = I.config(1)["dit"], 2, 1                 # configuration 1's draft pass, then its stand-alone pass
    elif which == "cfg2-bf16":
        dit, first, second = I.config(2)["dit"], 12, 4                # configuration 2's full pass (12 slots), then the solo one
    else:
        dit, first, second = dict(I.config(4)["dit"], depth=2, hidden=192, heads=3, lat_h=16, lat_w=16, cond_dim=64, ctx_len=9), 5, 2
    den = drf.Denoiser(dit, I.weights(dit, 11, "loud"))
    for k, slots in enumerate((first, second)):
        x, t, c = make(torch, dit, slots, 20 + k)
        want = den.eps_batched(x, t, c)
        got = torch.full_like(x, float("nan"))
        den.eps_batched_static(x, t, c, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (which, slots)
    den.close()


def test_static_scratch_entry_rejects_what_does_not_fit(torch, drf):
    dit = I.config(2)["dit"]
    den = drf.Denoiser(dit, I.weights(dit, 11))
    x, t, c = make(torch, dit, 64, 3)
    out = torch.zeros_like(x)
    with pytest.raises(drf.DrfError) as ei:
        den.eps_batched_static(x, t, c, out)                          # 64 slots need ~150 MB of scratch
    assert ei.value.status == -2                                      # DRF_ESHAPE, before any work is enqueued
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
    den.profile_enable(True)
    with pytest.raises(drf.DrfError):
        den.eps_batched_static(x[:2], t[:2], c[:2], out[:2])
    den.profile_enable(False)
    den.eps_batched_static(x[:2], t[:2], c[:2], out[:2])
    assert torch.equal(out[:2], den.eps_batched(x[:2], t[:2], c[:2]))
    den.close()


def test_static_scratch_entry_under_stream_capture(torch, drf):
    """One of the callers the entry point is for: the pass is recorded into a HIP graph (torch's capture of
    the stream the library is given) and replayed, with eager work and synchronisations between the replays;
    every replay must give the eager bits, also after the inputs changed in place."""
    dit = I.config(2, depth=3)["dit"]
    den = drf.Denoiser(dit, I.weights(dit, 12, "loud"))
    x, t, c = make(torch, dit, 6, 31)
    out = torch.empty_like(x)
    den.eps_batched_static(x, t, c, out)            # eager first: every kernel has been launched once
    want = den.eps_batched(x, t, c)
    x2 = torch.randn_like(x)
    want2 = den.eps_batched(x2, t, c)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    out.zero_()
    with torch.cuda.graph(graph):
        den.eps_batched_static(x, t, c, out)
    torch.cuda.synchronize()
    keep = x.clone()
    for it in range(4):
        if it % 2:
            x.copy_(x2)
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want2 if it % 2 else want), it
        x.copy_(keep)
        den.eps_batched(x2[:2], t[:2], c[:2])       # eager work on the handle's own workspace between replays
        torch.cuda.synchronize()
    den.close()
