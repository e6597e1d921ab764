"""Thin ctypes binding of libdrf's C ABI (see include/drf.h).

Argument marshalling only: torch supplies device buffers and the current HIP stream;
every step of the path runs in the library's kernels.  There is no CPU fallback: a
missing library raises at load."""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdrf.so")

CONSERVATIVE, AGGRESSIVE = 0, 1
F32, BF16 = 0, 1
COND_VECTOR, COND_CLASS, COND_TEXT = 0, 1, 2
PLAN_ROW = 5
PROF_GEMM, PROF_ATTN, PROF_ELEMWISE, PROF_UPDATE, PROF_PASS_FULL, PROF_PASS_OTHER = 0, 1, 2, 3, 4, 5
DDIM, DDPM, EULER = 0, 1, 2

# include/drf.h: the method's calls
SYMBOLS = ["drf_denoiser_weight_count", "drf_denoiser_create", "drf_denoiser_destroy", "drf_denoiser_reserve", "drf_denoiser_use_graphs",
           "drf_eps_batched", "drf_eps_batched_static", "drf_skip_transition", "drf_refine_step", "drf_sample",
           "drf_skip_transition_noise", "drf_normal_fill", "drf_sample_noise", "drf_noise_count",
           "drf_plan_build", "drf_last_error"]
# include/drf_measure.h: test and measurement hooks
MEASURE_SYMBOLS = ["drf_eps_trace", "drf_profile_enable", "drf_profile_read", "drf_probe_gemm_bf16",
                   "drf_probe_attn_bf16", "drf_probe_update_fused", "drf_graph_stats", "drf_calibrate_mfma_bf16", "drf_calibrate_copy"]
STATIC_SCRATCH_BYTES = 48 << 20


class DitConfig(C.Structure):
    _fields_ = [(k, C.c_int) for k in ("depth", "hidden", "heads", "mlp_ratio", "patch", "in_ch", "lat_h",
                                         "lat_w", "dtype", "cond", "cond_dim", "ctx_len")]


class SchedConfig(C.Structure):
    _fields_ = [("train_steps", C.c_int), ("beta_start", C.c_double), ("beta_end", C.c_double),
                ("steps", C.c_int), ("eta", C.c_double), ("sampler", C.c_int), ("shift", C.c_double)]


class Noise(C.Structure):
    _fields_ = [("z", C.c_void_p), ("seed", C.c_uint64), ("field0", C.c_uint32)]


class DrfError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("libdrf status %d: %s" % (status, msg))
        self.status = status


_lib = None


def lib():
    """Load libdrf.so (built by paper_2603_25872_amd/build.py); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libdrf.so is not built: run `python -m paper_2603_25872_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.drf_denoiser_weight_count.restype = C.c_size_t
        L.drf_denoiser_weight_count.argtypes = [C.c_void_p]
        L.drf_denoiser_create.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.drf_denoiser_destroy.argtypes = [C.c_void_p]
        L.drf_denoiser_destroy.restype = None
        L.drf_denoiser_reserve.argtypes = [C.c_void_p, C.c_int]
        L.drf_denoiser_use_graphs.argtypes = [C.c_void_p, C.c_int]
        L.drf_eps_batched.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.drf_eps_batched_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.drf_probe_update_fused.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float, C.c_size_t, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.drf_graph_stats.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.drf_calibrate_mfma_bf16.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.drf_calibrate_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.c_void_p]
        L.drf_eps_trace.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p,
                                    C.c_void_p]
        L.drf_skip_transition.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                          C.c_size_t, C.c_void_p, C.c_void_p]
        L.drf_refine_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_size_t, C.c_void_p,
                                      C.c_void_p]
        L.drf_sample.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                 C.c_void_p, C.c_float, C.c_void_p, C.c_void_p]
        L.drf_plan_build.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
        L.drf_skip_transition_noise.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                                C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p]
        L.drf_normal_fill.argtypes = [C.c_uint64, C.c_uint32, C.c_size_t, C.c_size_t, C.c_void_p, C.c_void_p]
        L.drf_sample_noise.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
        L.drf_noise_count.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.drf_profile_enable.argtypes = [C.c_void_p, C.c_int]
        L.drf_profile_read.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.drf_probe_gemm_bf16.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                          C.c_int, C.c_void_p]
        L.drf_probe_attn_bf16.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.drf_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        raise DrfError(status, lib().drf_last_error().decode())


def dit_config(d):
    return DitConfig(d["depth"], d["hidden"], d["heads"], d["mlp_ratio"], d["patch"], d["in_ch"], d["lat_h"],
                     d["lat_w"], d["dtype"], d["cond"], d["cond_dim"], d["ctx_len"])


def sched_config(d):
    return SchedConfig(d["train_steps"], d["beta_start"], d["beta_end"], d["steps"], float(d.get("eta", 0.0)),
                       int(d.get("sampler", DDIM)), float(d.get("shift", 1.0)))


def _noise(z=None, seed=None, field0=0):
    """drf_noise from explicit device fields z, or (seed, field0) of the library's stream; None when neither is given."""
    import torch
    if z is not None:
        return Noise(_dev(z, torch.float32), 0, 0)
    if seed is not None:
        return Noise(None, int(seed), int(field0))
    return None


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype=None):
    """Device pointer of a contiguous CUDA tensor."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "need a contiguous device tensor"
    if dtype is not None:
        assert t.dtype == dtype, "expected %s, got %s" % (dtype, t.dtype)
    return C.c_void_p(t.data_ptr())


def denoiser_weight_count(dit):
    cfg = dit_config(dit)
    return int(lib().drf_denoiser_weight_count(C.byref(cfg)))


def plan_build(sched, mode, n):
    """The bookkeeping table of drf_sample as an int32 array [rows, 5] (host only)."""
    sc = sched_config(sched)
    cnt = C.c_size_t(0)
    _check(lib().drf_plan_build(C.byref(sc), mode, n, None, 0, C.byref(cnt)))
    rows = np.zeros((cnt.value, PLAN_ROW), np.int32)
    _check(lib().drf_plan_build(C.byref(sc), mode, n, rows.ctypes.data_as(C.c_void_p), cnt.value, C.byref(cnt)))
    return rows


def skip_transition(sched, x_from, eps_from, s_from, s_to, out=None):
    """x_from, eps_from: fp32 device tensors [batch, ...]; s_to: list of target indices.
    Returns [len(s_to), batch, ...]."""
    import torch
    sc = sched_config(sched)
    m = len(s_to)
    batch = x_from.shape[0] if x_from.dim() > 0 else 1
    elems = x_from.numel() // batch if batch else 0
    if out is None:
        out = torch.empty((m,) + tuple(x_from.shape), dtype=torch.float32, device=x_from.device)
    tgt = (C.c_int * max(m, 1))(*s_to)
    _check(lib().drf_skip_transition(C.byref(sc), _dev(x_from, torch.float32), _dev(eps_from, torch.float32), s_from,
                                     tgt, m, batch, elems, _dev(out, torch.float32), _stream()))
    return out


def skip_transition_noise(sched, x_from, net_from, s_from, s_to, z=None, seed=None, field0=0, out=None):
    """Skip transitions of the configured sampler with their fresh noise: explicit fields z [len(s_to), batch, ...]
    or the library's stream (seed, field0)."""
    import torch
    sc = sched_config(sched)
    m = len(s_to)
    batch = x_from.shape[0] if x_from.dim() > 0 else 1
    elems = x_from.numel() // batch if batch else 0
    if out is None:
        out = torch.empty((m,) + tuple(x_from.shape), dtype=torch.float32, device=x_from.device)
    tgt = (C.c_int * max(m, 1))(*s_to)
    nz = _noise(z, seed, field0)
    _check(lib().drf_skip_transition_noise(C.byref(sc), _dev(x_from, torch.float32), _dev(net_from, torch.float32),
                                           s_from, tgt, m, batch, elems, C.byref(nz) if nz is not None else None,
                                           _dev(out, torch.float32), _stream()))
    return out


def normal_fill(seed, field0, n_fields, field_elems, out=None):
    """Fields field0 .. field0 + n_fields - 1 of the library's normal stream as a device tensor [n_fields, field_elems]."""
    import torch
    if out is None:
        out = torch.empty((n_fields, field_elems), dtype=torch.float32, device="cuda")
    _check(lib().drf_normal_fill(int(seed), int(field0), n_fields, field_elems, _dev(out, torch.float32), _stream()))
    return out


def noise_count(sched, mode, n):
    """Number of fresh-noise fields one drf_sample_noise call draws (host only)."""
    sc = sched_config(sched)
    cnt = C.c_size_t(0)
    _check(lib().drf_noise_count(C.byref(sc), mode, n, C.byref(cnt)))
    return int(cnt.value)


def refine_step(sched, x, eps, s_from, out=None):
    import torch
    sc = sched_config(sched)
    batch = x.shape[0]
    if out is None:
        out = torch.empty_like(x)
    _check(lib().drf_refine_step(C.byref(sc), _dev(x, torch.float32), _dev(eps, torch.float32), s_from, batch,
                                 x.numel() // batch if batch else 0, _dev(out, torch.float32), _stream()))
    return out


def probe_gemm_bf16(A, W, bias, out=None, variant=0):
    """out[M,N] = A[M,K] @ W[N,K]^T + bias with the library's bf16 GEMM (measurement hook)."""
    import torch
    M, K = A.shape
    N = W.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    _check(lib().drf_probe_gemm_bf16(_dev(A, torch.bfloat16), _dev(W, torch.bfloat16), M, N, K,
                                     _dev(out, torch.bfloat16), _dev(bias, torch.float32), variant, _stream()))
    return out


def probe_attn_bf16(qkv, slots, tokens, heads, head_dim, out=None):
    """Self-attention of the library on a packed bf16 [slots*tokens, 3*heads*head_dim] tensor (measurement hook)."""
    import torch
    if out is None:
        out = torch.empty((slots * tokens, heads * head_dim), dtype=torch.bfloat16, device=qkv.device)
    _check(lib().drf_probe_attn_bf16(_dev(qkv, torch.bfloat16), _dev(out, torch.bfloat16), slots, tokens, heads, head_dim,
                                     _stream()))
    return out


def probe_update_fused(sched, s_from, n_chain, n_draft, g, w, x_base, eps, x_out=None, draft_out=None):
    """One launch of the fused guidance + refine-chain + draft update kernel (measurement hook).
    x_base [field...], eps [max(n_chain,1), g, field...]; returns (x_out, draft_out [n_draft, field...])."""
    import torch
    sc = sched_config(sched)
    field = x_base.numel()
    if x_out is None:
        x_out = torch.empty_like(x_base)
    if draft_out is None and n_draft > 0:
        draft_out = torch.empty((n_draft,) + tuple(x_base.shape), dtype=torch.float32, device=x_base.device)
    _check(lib().drf_probe_update_fused(C.byref(sc), s_from, n_chain, n_draft, g, float(w), field, _dev(x_base, torch.float32),
                                        _dev(eps, torch.float32), _dev(x_out, torch.float32), _dev(draft_out, torch.float32),
                                        _stream()))
    return x_out, draft_out


def calibrate_mfma_bf16(random_operands=True, iters=5):
    """TFLOP/s of a loop of nothing but the GEMM kernel's MFMA instruction on this GPU (measurement hook)."""
    v = C.c_double(0)
    _check(lib().drf_calibrate_mfma_bf16(1 if random_operands else 0, iters, C.byref(v), _stream()))
    return v.value


def calibrate_copy(src, dst, iters=5):
    """GB/s (read + written) of a plain copy kernel between two device tensors of equal size (measurement hook)."""
    v = C.c_double(0)
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib().drf_calibrate_copy(_dev(src), _dev(dst), nbytes, iters, C.byref(v), _stream()))
    return v.value


class Denoiser:
    """Owns a drf_denoiser handle."""

    def __init__(self, dit, host_weights):
        self.dit = dict(dit)
        w = np.ascontiguousarray(host_weights, np.float32)
        cfg = dit_config(dit)
        h = C.c_void_p()
        _check(lib().drf_denoiser_create(C.byref(cfg), w.ctypes.data_as(C.c_void_p), w.size, _stream(), C.byref(h)))
        self.h = h

    def close(self):
        h, self.h = getattr(self, "h", None), None
        if h and _lib is not None:              # at interpreter exit the module may already be torn down
            _lib.drf_denoiser_destroy(h)

    __del__ = close

    def reserve(self, max_slots):
        _check(lib().drf_denoiser_reserve(self.h, max_slots))

    def use_graphs(self, mode):
        """0: sample() launches kernel by kernel; 1 (default): replays a captured graph from the second identical
        call on; 2: captures at the first call."""
        _check(lib().drf_denoiser_use_graphs(self.h, int(mode)))

    def graph_stats(self):
        a, b, c = C.c_int(0), C.c_int(0), C.c_longlong(0)
        _check(lib().drf_graph_stats(self.h, C.byref(a), C.byref(b), C.byref(c)))
        return dict(captured=a.value, failed=b.value, replays=c.value)

    def _cond_dtype(self):
        import torch
        return torch.int32 if self.dit["cond"] == COND_CLASS else torch.float32

    def eps_batched(self, x, t, cond, out=None):
        import torch
        if out is None:
            out = torch.empty_like(x)
        _check(lib().drf_eps_batched(self.h, _dev(x, torch.float32), _dev(t, torch.int32),
                                     _dev(cond, self._cond_dtype()), x.shape[0], _dev(out, torch.float32), _stream()))
        return out

    def eps_batched_static(self, x, t, cond, out):
        """drf_eps_batched on the library's static scratch array: the call allocates nothing, so `out` is required."""
        import torch
        _check(lib().drf_eps_batched_static(self.h, _dev(x, torch.float32), _dev(t, torch.int32),
                                            _dev(cond, self._cond_dtype()), x.shape[0], _dev(out, torch.float32), _stream()))
        return out

    def eps_trace(self, x, t, cond, n_blocks):
        import torch
        d = self.dit
        T = (d["lat_h"] // d["patch"]) * (d["lat_w"] // d["patch"])
        out = torch.empty((x.shape[0], T, d["hidden"]), dtype=torch.float32, device=x.device)
        _check(lib().drf_eps_trace(self.h, _dev(x, torch.float32), _dev(t, torch.int32),
                                   _dev(cond, self._cond_dtype()), x.shape[0], n_blocks, _dev(out), _stream()))
        return out

    def sample(self, sched, mode, n, x_T, cond, null_cond=None, cfg_scale=0.0, out=None):
        import torch
        sc = sched_config(sched)
        if out is None:
            out = torch.empty_like(x_T)
        _check(lib().drf_sample(self.h, C.byref(sc), mode, n, x_T.shape[0], _dev(x_T, torch.float32),
                                _dev(cond, self._cond_dtype()), _dev(null_cond, self._cond_dtype()),
                                float(cfg_scale or 0.0), _dev(out, torch.float32), _stream()))
        return out

    def sample_noise(self, sched, mode, n, x_T, cond, null_cond=None, cfg_scale=0.0, z=None, seed=None, field0=0,
                     out=None):
        import torch
        sc = sched_config(sched)
        if out is None:
            out = torch.empty_like(x_T)
        nz = _noise(z, seed, field0)
        _check(lib().drf_sample_noise(self.h, C.byref(sc), mode, n, x_T.shape[0], _dev(x_T, torch.float32),
                                      _dev(cond, self._cond_dtype()), _dev(null_cond, self._cond_dtype()),
                                      float(cfg_scale or 0.0), C.byref(nz) if nz is not None else None,
                                      _dev(out, torch.float32), _stream()))
        return out

    def profile_enable(self, on=1):
        """0 off, 1 (True) per launch, 2 per predictor pass of sample()"""
        _check(lib().drf_profile_enable(self.h, int(on)))

    def profile_read(self, which):
        n, ms, work = C.c_longlong(0), C.c_double(0), C.c_double(0)
        _check(lib().drf_profile_read(self.h, which, C.byref(n), C.byref(ms), C.byref(work)))
        return dict(launches=n.value, ms=ms.value, work=work.value)
