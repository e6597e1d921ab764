"""Host-side checks that need no GPU: the library loads, exports every symbol the
header declares, its plan table equals the oracle's bit for bit, and bad arguments
come back as status codes."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2603_25872_amd import drf, inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols(name):
    text = open(os.path.join(ROOT, "include", name)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(drf_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = drf.lib()
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["drf.h", "drf_measure.h"]
    assert header_symbols("drf.h") == sorted(drf.SYMBOLS)
    assert header_symbols("drf_measure.h") == sorted(drf.MEASURE_SYMBOLS)
    for n in drf.SYMBOLS + drf.MEASURE_SYMBOLS:
        assert getattr(L, n) is not None
    # the measurement hooks stay out of the method's header
    assert not set(drf.MEASURE_SYMBOLS) & set(header_symbols("drf.h"))


def sched(S):
    return dict(train_steps=1000, beta_start=1e-4, beta_end=0.02, steps=S, eta=0.0)


@pytest.mark.parametrize("mode", [drf.CONSERVATIVE, drf.AGGRESSIVE])
@pytest.mark.parametrize("S", [1, 2, 3, 5, 20, 28, 30, 50, 1000])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 8, 9, 64, 100])
def test_plan_table_bit_exact_with_oracle(orc, mode, S, n):
    got = drf.plan_build(sched(S), mode, n)
    want = orc.plan(sched(S), mode, n)
    assert got.dtype == want.dtype == np.int32
    assert got.shape == want.shape
    assert np.array_equal(got, want)


def test_plan_for_the_five_workloads(orc):
    for idx, c in I.CONFIGS.items():
        assert np.array_equal(drf.plan_build(c["sched"], c["mode"], c["n"]), orc.plan(c["sched"], c["mode"], c["n"]))


def test_plan_capacity_is_respected():
    sc = drf.sched_config(sched(20))
    cnt = C.c_size_t(0)
    rows = np.full((3, 5), -7, np.int32)
    assert drf.lib().drf_plan_build(C.byref(sc), 0, 2, rows.ctypes.data_as(C.c_void_p), 2, C.byref(cnt)) == 0
    assert cnt.value > 3
    assert (rows[2] == -7).all() and (rows[:2] != -7).any()


@pytest.mark.parametrize("bad", [dict(steps=0), dict(steps=1001), dict(eta=1.5), dict(eta=-0.1), dict(beta_start=0.0),
                                 dict(beta_end=1.0), dict(train_steps=1), dict(sampler=3), dict(sampler=-1),
                                 dict(sampler=drf.EULER, shift=0.0)])
def test_bad_schedule_is_a_status_code(bad):
    sc = drf.sched_config(dict(sched(20), **bad))
    cnt = C.c_size_t(0)
    st = drf.lib().drf_plan_build(C.byref(sc), 0, 2, None, 0, C.byref(cnt))
    assert st == -1
    assert len(drf.lib().drf_last_error()) > 0


@pytest.mark.parametrize("mode", [drf.CONSERVATIVE, drf.AGGRESSIVE])
@pytest.mark.parametrize("S", [1, 2, 3, 7, 28, 50])
@pytest.mark.parametrize("n", [1, 2, 4, 9])
@pytest.mark.parametrize("extra", [dict(eta=1.0), dict(sampler=drf.DDPM), dict(sampler=drf.EULER),
                                   dict(sampler=drf.EULER, shift=3.0)])
def test_plan_and_draw_count_of_the_other_samplers(orc, mode, S, n, extra):
    sd = dict(sched(S), **extra)
    got = drf.plan_build(sd, mode, n)
    assert np.array_equal(got, orc.plan(sd, mode, n))
    assert drf.noise_count(sd, mode, n) == orc.noise_count(sd, mode, n) == int((got[:, 1] != 0).sum())


def test_euler_plan_feeds_sigma_scaled_times(orc):
    sd = dict(sched(28), sampler=drf.EULER, shift=3.0)
    rows = drf.plan_build(sd, drf.CONSERVATIVE, 4)
    evald = rows[rows[:, 4] >= 0]
    for r in evald:
        u = r[3] / 28
        assert r[4] == int(np.floor(3 * u / (1 + 2 * u) * 1000 + 0.5))
    assert evald[0, 4] == 1000


def test_stochastic_sampler_without_noise_source_is_rejected_before_any_launch():
    # validation happens on the host: fake (never dereferenced) device addresses are enough
    L = drf.lib()
    fake = C.c_void_p(0x1000)
    to = (C.c_int * 2)(4, 3)
    for extra in (dict(eta=0.5), dict(sampler=drf.DDPM)):
        sc = drf.sched_config(dict(sched(20), **extra))
        assert L.drf_skip_transition_noise(C.byref(sc), fake, fake, 5, to, 2, 1, 16, None, fake, None) == -1
        assert b"noise source" in L.drf_last_error()
        assert L.drf_skip_transition(C.byref(sc), fake, fake, 5, to, 2, 1, 16, fake, None) == -1
        # a transition with variance has to move towards data
        up = (C.c_int * 1)(7)
        nz = drf.Noise(None, 1, 0)
        assert L.drf_skip_transition_noise(C.byref(sc), fake, fake, 5, up, 1, 1, 16, C.byref(nz), fake, None) == -1
        assert b"towards data" in L.drf_last_error()
    cnt = C.c_size_t(0)
    sc = drf.sched_config(sched(20))
    assert L.drf_noise_count(C.byref(sc), 0, 2, None) == -1
    assert L.drf_noise_count(C.byref(sc), 0, 0, C.byref(cnt)) == -1
    assert L.drf_normal_fill(1, 0, 4, 16, None, None) == -1
    assert L.drf_normal_fill(1, 0, 0, 16, None, None) == 0
    assert L.drf_normal_fill(1, 0xffffffff, 2, 16, fake, None) == -1


def test_bad_plan_arguments():
    sc = drf.sched_config(sched(20))
    cnt = C.c_size_t(0)
    L = drf.lib()
    assert L.drf_plan_build(C.byref(sc), 0, 0, None, 0, C.byref(cnt)) == -1
    assert L.drf_plan_build(C.byref(sc), 5, 2, None, 0, C.byref(cnt)) == -1
    assert L.drf_plan_build(None, 0, 2, None, 0, C.byref(cnt)) == -1
    assert L.drf_plan_build(C.byref(sc), 0, 2, None, 0, None) == -1


def test_weight_count_matches_layout_and_oracle(orc):
    for idx, c in I.CONFIGS.items():
        n = drf.denoiser_weight_count(c["dit"])
        assert n == I.param_count(c["dit"]) == orc.weight_count(c["dit"])
    assert drf.denoiser_weight_count(dict(I.CONFIGS[1]["dit"], hidden=130)) == 0       # not divisible by heads
    assert drf.denoiser_weight_count(dict(I.CONFIGS[2]["dit"], hidden=390)) == 0       # bf16 needs % 64


def test_null_handles_are_rejected_without_touching_the_gpu():
    L = drf.lib()
    assert L.drf_eps_batched(None, None, None, None, 1, None, None) == -1
    assert L.drf_sample(None, None, 0, 1, 1, None, None, None, C.c_float(0), None, None) == -1
    assert L.drf_denoiser_reserve(None, 4) == -1
    L.drf_denoiser_destroy(None)
    sc = drf.sched_config(sched(20))
    to = (C.c_int * 1)(3)
    # zero-sized work is a no-op, NULL buffers with real sizes are an error
    assert L.drf_skip_transition(C.byref(sc), None, None, 5, to, 1, 0, 16, None, None) == 0
    assert L.drf_skip_transition(C.byref(sc), None, None, 5, to, 1, 2, 16, None, None) == -1
    assert L.drf_refine_step(C.byref(sc), None, None, 0, 1, 16, None, None) == -1
    # the entry point that allocates nothing, the graph switch and the measurement hooks
    assert L.drf_eps_batched_static(None, None, None, None, 1, None, None) == -1
    assert L.drf_denoiser_use_graphs(None, 1) == -1
    a, b, c = C.c_int(0), C.c_int(0), C.c_longlong(0)
    assert L.drf_graph_stats(None, C.byref(a), C.byref(b), C.byref(c)) == -1
    assert L.drf_profile_enable(None, 1) == -1
    v = C.c_double(0)
    assert L.drf_calibrate_mfma_bf16(1, 0, C.byref(v), None) == -1           # iters < 1
    assert L.drf_calibrate_copy(None, None, 1024, 1, C.byref(v), None) == -1
    # the fused-update probe validates its counts and indices on the host before any launch
    assert L.drf_probe_update_fused(C.byref(sc), 20, 4, 4, 3, C.c_float(1), 16, None, None, None, None, None) == -1   # g not 1 | 2
    assert L.drf_probe_update_fused(C.byref(sc), 5, 4, 4, 2, C.c_float(1), 16, None, None, None, None, None) == -1    # runs past index 0
    assert L.drf_probe_update_fused(C.byref(sc), 20, 4, 4, 2, C.c_float(1), 0, None, None, None, None, None) == 0     # empty field: no-op
    assert L.drf_probe_update_fused(C.byref(sc), 20, 4, 4, 2, C.c_float(1), 16, None, None, None, None, None) == -1   # NULL buffers
    assert len(L.drf_last_error()) > 0


def test_bench_refuses_more_than_one_gpu():
    # the contract: bench.py --gpus N with N > 1 exits with a message that says so (no GPU is touched)
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
