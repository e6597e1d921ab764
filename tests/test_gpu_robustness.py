"""Failure handling of the handle on the GPU machine: a failed workspace allocation leaves the handle usable,
and a second handle cannot put work in flight beside a running one."""
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


def small(dtype, **kw):
    base = dict(depth=2, hidden=128, heads=4, mlp_ratio=4, patch=2, in_ch=4, lat_h=10, lat_w=6, dtype=dtype,
                cond=I.COND_CLASS, cond_dim=10, ctx_len=0)
    base.update(kw)
    return base


@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
def test_failed_allocation_leaves_the_handle_usable(torch, drf, dtype):
    dit = small(dtype)
    den = drf.Denoiser(dit, I.weights(dit, 9))
    x = torch.randn((3, 4, 10, 6), device="cuda")
    t = torch.tensor([1, 500, 999], dtype=torch.int32, device="cuda")
    c = torch.tensor([0, 5, 10], dtype=torch.int32, device="cuda")
    before = den.eps_batched(x, t, c)
    with pytest.raises(drf.DrfError) as ei:
        den.reserve(2 ** 31 - 1)                     # tens of terabytes
    assert ei.value.status == -3                     # DRF_ENOMEM
    # every workspace pointer is NULL or live again: the next calls re-allocate and give the same bits
    assert torch.equal(before, den.eps_batched(x, t, c))
    with pytest.raises(drf.DrfError):
        den.reserve(2 ** 31 - 1)
    sd = dict(train_steps=1000, beta_start=1e-4, beta_end=0.02, steps=4, eta=0.0)
    y = den.sample(sd, I.AGGRESSIVE, 2, x, c)
    assert bool(torch.isfinite(y).all())
    assert torch.equal(before, den.eps_batched(x, t, c))
    den.close()


def test_second_handle_is_refused_while_the_first_is_in_flight(torch, drf):
    """Only one handle may have work in flight: a call on another handle from another stream while the first
    handle's work is still running returns DRF_EUNSUPPORTED before anything is enqueued, and works after a
    synchronisation.  (No two handles ever run at the same time here.)"""
    dit = small(I.BF16, depth=6, hidden=1152, heads=16, lat_h=32, lat_w=32)
    w = I.weights(dit, 9)
    a, b = drf.Denoiser(dit, w), drf.Denoiser(dit, w)
    slots = 128                                      # ~6.5 TFLOP per pass: several milliseconds on the GPU
    x = torch.randn((slots, 4, 32, 32), device="cuda")
    t = torch.randint(0, 1000, (slots,), dtype=torch.int32, device="cuda")
    c = torch.randint(0, 11, (slots,), dtype=torch.int32, device="cuda")
    a.reserve(slots)
    b.reserve(2)
    out_a = torch.empty_like(x)
    out_b = torch.empty_like(x[:2])
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    a.eps_batched(x, t, c, out=out_a)                # several milliseconds of GPU work, enqueued in well under one
    refused = False
    with torch.cuda.stream(side):
        try:
            b.eps_batched(x[:2], t[:2], c[:2], out=out_b)
        except drf.DrfError as e:
            refused = True
            assert e.status == -5                    # DRF_EUNSUPPORTED
    torch.cuda.synchronize()
    assert refused, "the first handle's pass should still have been running"
    # same stream: stream order serialises the two handles, so this is allowed
    a.eps_batched(x, t, c, out=out_a)
    b.eps_batched(x[:2], t[:2], c[:2], out=out_b)
    torch.cuda.synchronize()

    def same_slots(small, big):
        # a 2-slot pass and the first slots of a 128-slot pass: the same values up to the order of the GEMMs' k-sums
        # (tile shapes, and the split of K across workgroups for few-tile problems, depend on the number of rows)
        return float((small - big).abs().max() / big.abs().max()) < 5e-3

    assert same_slots(out_b, out_a[:2])
    first = out_b.clone()
    # other stream after a synchronisation: allowed
    with torch.cuda.stream(side):
        b.eps_batched(x[:2], t[:2], c[:2], out=out_b)
    torch.cuda.synchronize()
    assert torch.equal(out_b, first)                 # the same call again: bit for bit
    # the same handle on another stream while its own work is still running: refused as well
    a.eps_batched(x, t, c, out=out_a)
    moved = False
    with torch.cuda.stream(side):
        try:
            a.eps_batched(x[:2], t[:2], c[:2], out=out_b)
        except drf.DrfError as e:
            moved = e.status == -5
    torch.cuda.synchronize()
    assert moved
    a.close(); b.close()


def test_more_slots_than_a_launch_covers_is_a_status_code(torch, drf):
    """Some launches index slots by a grid dimension, so a pass is limited to 65535 slots: beyond that the call
    returns DRF_ESHAPE before anything is enqueued."""
    dit = small(I.F32, depth=1, lat_h=2, lat_w=2)
    den = drf.Denoiser(dit, I.weights(dit, 9))
    slots = 65536
    x = torch.zeros((slots, 4, 2, 2), device="cuda")
    t = torch.zeros((slots,), dtype=torch.int32, device="cuda")
    out = torch.full_like(x, 7.0)
    with pytest.raises(drf.DrfError) as ei:
        den.eps_batched(x, t, t, out=out)
    assert ei.value.status == -2
    torch.cuda.synchronize()
    assert float(out.min()) == 7.0
    sd = dict(train_steps=1000, beta_start=1e-4, beta_end=0.02, steps=4, eta=0.0)
    with pytest.raises(drf.DrfError) as ei:
        den.sample(sd, I.AGGRESSIVE, 2, x[:40000], t[:40000])          # 2 groups x 40000 slots per pass
    assert ei.value.status == -2
    ok = den.eps_batched(x[:65535], t[:65535], t[:65535])
    assert bool(torch.isfinite(ok).all())
    den.close()
