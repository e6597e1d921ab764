"""ctypes front for the C oracle (TEST INFRASTRUCTURE ONLY -- never imported by the
product package).  All method arithmetic lives in drf_oracle.c; this file only
marshals numpy arrays."""
import ctypes as C
import os

import numpy as np

from . import build as _build

ROW = 5


class Sched(C.Structure):
    _fields_ = [("train_steps", C.c_int), ("beta_start", C.c_double), ("beta_end", C.c_double),
                ("steps", C.c_int), ("eta", C.c_double), ("sampler", C.c_int), ("shift", C.c_double)]


class DitConfig(C.Structure):
    _fields_ = [(k, C.c_int) for k in ("depth", "hidden", "heads", "mlp_ratio", "patch", "in_ch",
                                         "lat_h", "lat_w", "cond_kind", "cond_dim", "ctx_len",
                                         "round_bf16")]


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


class Oracle:
    """bits=64: double arithmetic (authority). bits=32: float build of the same source."""

    def __init__(self, bits=64):
        _build.build()
        self.lib = C.CDLL(_build.lib_path(bits))
        self.real = np.float64 if bits == 64 else np.float32
        assert self.lib.orc_real_bytes() == bits // 8
        L = self.lib
        L.orc_weight_count.restype = C.c_size_t
        L.orc_abar_at.restype = C.c_double
        L.orc_skip.argtypes = [C.c_void_p, C.c_void_p, C.c_double, C.c_double, C.c_size_t, C.c_void_p]
        self.EPS_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p)
        L.orc_sample.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_size_t, C.c_void_p, C.c_void_p,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.orc_sigma_at.restype = C.c_double
        L.orc_posterior_var.restype = C.c_double
        L.orc_posterior_var.argtypes = [C.c_double, C.c_double]
        L.orc_sigma.restype = C.c_double
        L.orc_sigma.argtypes = [C.c_double, C.c_double, C.c_double]
        L.orc_skip_eta.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_double, C.c_double, C.c_double,
                                   C.c_size_t, C.c_void_p]
        L.orc_ddpm_skip.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_double, C.c_double, C.c_size_t,
                                    C.c_void_p]
        L.orc_euler_skip.argtypes = [C.c_void_p, C.c_void_p, C.c_double, C.c_double, C.c_size_t, C.c_void_p]
        L.orc_noise_count.restype = C.c_long
        L.orc_normal_fill.argtypes = [C.c_uint64, C.c_uint32, C.c_size_t, C.c_size_t, C.c_void_p]
        L.orc_dit_eps.argtypes = [C.c_void_p] * 5 + [C.c_int, C.c_void_p, C.c_int, C.c_void_p]
        L.orc_sample_dit.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_double, C.c_void_p]
        L.orc_eps_guided.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                     C.c_void_p, C.c_double, C.c_int, C.c_void_p]

    def linear(self, x, W, b):
        """y = x W^T + b with the oracle's plain triple loop."""
        x = np.ascontiguousarray(x, self.real); W = np.ascontiguousarray(W, self.real)
        b = np.ascontiguousarray(b, self.real)
        M, K = x.shape
        N = W.shape[0]
        y = np.empty((M, N), self.real)
        self.lib.orc_linear.argtypes = [C.c_void_p] * 4 + [C.c_size_t] * 3
        self.lib.orc_linear(_ptr(y), _ptr(x), _ptr(W), _ptr(b), M, K, N)
        return y

    def attention_packed(self, qkv, tokens, heads, d):
        """Self-attention per slot on packed rows [slots*tokens, 3*heads*d] (q | k | v)."""
        qkv = np.ascontiguousarray(qkv, self.real)
        D = heads * d
        slots = qkv.shape[0] // tokens
        out = np.empty((slots * tokens, D), self.real)
        self.lib.orc_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_size_t,
                                           C.c_size_t, C.c_size_t, C.c_int, C.c_size_t]
        item = qkv.itemsize
        for s in range(slots):
            base = qkv.ctypes.data + s * tokens * 3 * D * item
            self.lib.orc_attention(C.c_void_p(out.ctypes.data + s * tokens * D * item), C.c_void_p(base), 3 * D,
                                   C.c_void_p(base + D * item), C.c_void_p(base + 2 * D * item), 3 * D, tokens, tokens,
                                   heads, d)
        return out

    def threads(self):
        return int(self.lib.orc_num_threads())

    # ---- schedule
    @staticmethod
    def sched(d):
        return Sched(d["train_steps"], d["beta_start"], d["beta_end"], d["steps"], float(d.get("eta", 0.0)),
                     int(d.get("sampler", 0)), float(d.get("shift", 1.0)))

    def alpha_bar(self, sd):
        sc = self.sched(sd)
        out = np.empty(sd["train_steps"], np.float64)
        self.lib.orc_alpha_bar(C.byref(sc), _ptr(out))
        return out

    def tau(self, sd, s):
        sc = self.sched(sd)
        return int(self.lib.orc_tau(C.byref(sc), C.c_int(s)))

    def abar_at(self, sd, s):
        ab = self.alpha_bar(sd)
        sc = self.sched(sd)
        return float(self.lib.orc_abar_at(C.byref(sc), _ptr(ab), C.c_int(s)))

    def sigma_at(self, sd, s):
        sc = self.sched(sd)
        return float(self.lib.orc_sigma_at(C.byref(sc), C.c_int(s)))

    def net_time(self, sd, s):
        sc = self.sched(sd)
        return int(self.lib.orc_net_time(C.byref(sc), C.c_int(s)))

    # ---- operator
    def skip(self, x, eps, a_from, a_to):
        x = np.ascontiguousarray(x, self.real)
        eps = np.ascontiguousarray(eps, self.real)
        out = np.empty_like(x)
        self.lib.orc_skip(_ptr(x), _ptr(eps), a_from, a_to, x.size, _ptr(out))
        return out

    def posterior_var(self, a_from, a_to):
        return float(self.lib.orc_posterior_var(a_from, a_to))

    def sigma(self, eta, a_from, a_to):
        return float(self.lib.orc_sigma(eta, a_from, a_to))

    def _z(self, z, like):
        if z is None:
            return None
        z = np.ascontiguousarray(z, self.real)
        return z

    def skip_eta(self, x, eps, z, a_from, a_to, sigma):
        x = np.ascontiguousarray(x, self.real)
        eps = np.ascontiguousarray(eps, self.real)
        z = self._z(z, x)
        out = np.empty_like(x)
        self.lib.orc_skip_eta(_ptr(x), _ptr(eps), _ptr(z), a_from, a_to, sigma, x.size, _ptr(out))
        return out

    def ddpm_skip(self, x, eps, z, a_from, a_to):
        x = np.ascontiguousarray(x, self.real)
        eps = np.ascontiguousarray(eps, self.real)
        z = self._z(z, x)
        out = np.empty_like(x)
        self.lib.orc_ddpm_skip(_ptr(x), _ptr(eps), _ptr(z), a_from, a_to, x.size, _ptr(out))
        return out

    def euler_skip(self, x, v, sig_from, sig_to):
        x = np.ascontiguousarray(x, self.real)
        v = np.ascontiguousarray(v, self.real)
        out = np.empty_like(x)
        self.lib.orc_euler_skip(_ptr(x), _ptr(v), sig_from, sig_to, x.size, _ptr(out))
        return out

    # ---- noise stream
    def philox(self, ctr, key):
        c = (C.c_uint32 * 4)(*ctr)
        k = (C.c_uint32 * 2)(*key)
        o = (C.c_uint32 * 4)()
        self.lib.orc_philox4x32(c, k, o)
        return [int(v) for v in o]

    def normal_fill(self, seed, field0, n_fields, F):
        out = np.empty((n_fields, F), self.real)
        self.lib.orc_normal_fill(C.c_uint64(seed), C.c_uint32(field0), n_fields, F, _ptr(out))
        return out

    def noise_count(self, sd, mode, n):
        sc = self.sched(sd)
        return int(self.lib.orc_noise_count(C.byref(sc), mode, n))

    # ---- scheduler
    def plan(self, sd, mode, n):
        sc = self.sched(sd)
        cnt = C.c_size_t(0)
        rc = self.lib.orc_sample(C.byref(sc), mode, n, 0, 0, None, None, None, None, None, None, 0, C.byref(cnt))
        if rc != 0:
            raise ValueError("oracle rejected plan arguments")
        rows = np.zeros((cnt.value, ROW), np.int32)
        self.lib.orc_sample(C.byref(sc), mode, n, 0, 0, None, None, None, None, None, _ptr(rows), cnt.value,
                            C.byref(cnt))
        return rows

    def sample_with(self, sd, mode, n, xT, eps_py, z=None):
        """Run the scheduler with a Python noise predictor eps_py(x, s, tau) -> eps,
        x shaped like xT ([batch, ...]); z: noise fields [n_noise, batch, ...] or None."""
        xT = np.ascontiguousarray(xT, self.real)
        if z is not None:
            z = np.ascontiguousarray(z, self.real)
            assert z.shape[0] >= self.noise_count(sd, mode, n) and z[0].size == xT.size
        batch = xT.shape[0]
        E = xT.size // batch
        shape = xT.shape
        real = self.real

        def cb(user, xp, s, tau, outp):
            x = np.frombuffer((C.c_char * xT.nbytes).from_address(xp), dtype=real).reshape(shape)
            out = np.frombuffer((C.c_char * xT.nbytes).from_address(outp), dtype=real).reshape(shape)
            out[...] = eps_py(x.copy(), s, tau)

        fn = self.EPS_FN(cb)
        x0 = np.empty_like(xT)
        sc = self.sched(sd)
        rc = self.lib.orc_sample(C.byref(sc), mode, n, batch, E, _ptr(xT), _ptr(z), C.cast(fn, C.c_void_p), None,
                                 _ptr(x0), None, 0, None)
        if rc != 0:
            raise ValueError("oracle rejected sample arguments")
        return x0

    # ---- DiT
    @staticmethod
    def dit_config(d):
        return DitConfig(d["depth"], d["hidden"], d["heads"], d["mlp_ratio"], d["patch"], d["in_ch"],
                         d["lat_h"], d["lat_w"], d["cond"], d["cond_dim"], d["ctx_len"],
                         1 if d["dtype"] == 1 else 0)

    def weight_count(self, d):
        cfg = self.dit_config(d)
        return int(self.lib.orc_weight_count(C.byref(cfg)))

    def _cond(self, d, cond):
        if cond is None:
            return None
        if d["cond"] == 1:
            return np.ascontiguousarray(cond, np.int32)
        return np.ascontiguousarray(cond, self.real)

    def prepare_weights(self, w):
        """Convert the flat fp32 weights to the oracle's real type once."""
        return np.ascontiguousarray(w, self.real)

    def dit_eps(self, d, w, x, t, cond, stop_blocks=-1):
        cfg = self.dit_config(d)
        w = self.prepare_weights(w)
        assert w.size == self.weight_count(d)
        x = np.ascontiguousarray(x, self.real)
        t = np.ascontiguousarray(t, np.int32)
        slots = x.shape[0]
        cond = self._cond(d, cond)
        if stop_blocks >= 0:
            T = (d["lat_h"] // d["patch"]) * (d["lat_w"] // d["patch"])
            res = np.empty((slots, T, d["hidden"]), self.real)
            rc = self.lib.orc_dit_eps(C.byref(cfg), _ptr(w), _ptr(x), _ptr(t), _ptr(cond), slots, None,
                                      stop_blocks, _ptr(res))
            assert rc == 0
            return res
        out = np.empty_like(x)
        rc = self.lib.orc_dit_eps(C.byref(cfg), _ptr(w), _ptr(x), _ptr(t), _ptr(cond), slots, _ptr(out),
                                  -1, None)
        assert rc == 0
        return out

    def eps_guided(self, d, w, x, tau, cond, null_cond, guidance):
        cfg = self.dit_config(d)
        w = self.prepare_weights(w)
        x = np.ascontiguousarray(x, self.real)
        out = np.empty_like(x)
        cond, null_cond = self._cond(d, cond), self._cond(d, null_cond)
        self.lib.orc_eps_guided(C.byref(cfg), _ptr(w), _ptr(x), tau, _ptr(cond), _ptr(null_cond),
                                float(guidance or 0.0), x.shape[0], _ptr(out))
        return out

    def sample_dit(self, d, w, sd, mode, n, xT, cond, null_cond=None, guidance=0.0, z=None):
        cfg = self.dit_config(d)
        w = self.prepare_weights(w)
        xT = np.ascontiguousarray(xT, self.real)
        x0 = np.empty_like(xT)
        sc = self.sched(sd)
        cond, null_cond = self._cond(d, cond), self._cond(d, null_cond)
        if z is not None:
            z = np.ascontiguousarray(z, self.real)
            assert z.shape[0] >= self.noise_count(sd, mode, n) and z[0].size == xT.size
        rc = self.lib.orc_sample_dit(C.byref(cfg), _ptr(w), C.byref(sc), mode, n, xT.shape[0], _ptr(xT), _ptr(z),
                                     _ptr(cond), _ptr(null_cond), float(guidance or 0.0), _ptr(x0))
        if rc != 0:
            raise ValueError("oracle rejected sample arguments")
        return x0
