"""Seeded synthetic inputs for the DRiffusion hot path.

This module holds none of the method's arithmetic: it only names the workload
configurations, lists parameter tensors in the canonical order of the flat weight
array (an interface both the library and the test oracle implement on their own),
and draws seeded random numbers with numpy's counter-based Philox generator.
The tensors stand in for the pretrained Stable-Diffusion weights and MS-COCO
captions of the paper's experiment section, which are not available here.
"""
import numpy as np

BASE_SEED = 2603025872

COND_VECTOR, COND_CLASS, COND_TEXT = 0, 1, 2
CONSERVATIVE, AGGRESSIVE = 0, 1
F32, BF16 = 0, 1
TFREQ = 256


def _dit(depth, hidden, heads, lat, dtype, cond, cond_dim, ctx_len=0):
    return dict(depth=depth, hidden=hidden, heads=heads, mlp_ratio=4, patch=2, in_ch=4,
                lat_h=lat, lat_w=lat, dtype=dtype, cond=cond, cond_dim=cond_dim, ctx_len=ctx_len)


def _sched(steps):
    return dict(train_steps=1000, beta_start=1e-4, beta_end=0.02, steps=steps, eta=0.0)


# The five workload configurations (index 1..5).
CONFIGS = {
    1: dict(name="tiny-dit-f32", dit=_dit(2, 128, 4, 16, F32, COND_VECTOR, 128), sched=_sched(20),
            mode=CONSERVATIVE, n=2, batch=1, guidance=None),
    2: dict(name="dit-s-bf16", dit=_dit(12, 384, 6, 32, BF16, COND_CLASS, 1000), sched=_sched(50),
            mode=AGGRESSIVE, n=3, batch=4, guidance=None),
    3: dict(name="dit-xl2-bf16-cfg4", dit=_dit(28, 1152, 16, 32, BF16, COND_CLASS, 1000), sched=_sched(50),
            mode=CONSERVATIVE, n=4, batch=8, guidance=4.0),
    4: dict(name="text-dit-bf16-cfg7", dit=_dit(28, 1152, 16, 128, BF16, COND_TEXT, 1024, 77),
            sched=_sched(30), mode=AGGRESSIVE, n=3, batch=1, guidance=7.0),
    5: dict(name="wide-draft-bf16-cfg4", dit=_dit(28, 1152, 16, 64, BF16, COND_CLASS, 1000), sched=_sched(50),
            mode=CONSERVATIVE, n=8, batch=4, guidance=4.0),
}


def config(idx, **dit_overrides):
    """A deep copy of configuration `idx`, with DiT fields optionally overridden
    (e.g. depth=2 for a reduced-depth parity case)."""
    c = CONFIGS[idx]
    out = dict(c)
    out["dit"] = dict(c["dit"], **dit_overrides)
    out["sched"] = dict(c["sched"])
    return out


def param_shapes(dit):
    """(name, shape) of every parameter tensor in flat-array order; Linear weights
    are [out, in]."""
    D, R = dit["hidden"], dit["mlp_ratio"]
    P = dit["in_ch"] * dit["patch"] ** 2
    out = [("patch_w", (D, P)), ("patch_b", (D,)),
           ("t_w1", (D, TFREQ)), ("t_b1", (D,)), ("t_w2", (D, D)), ("t_b2", (D,))]
    if dit["cond"] == COND_VECTOR:
        out += [("c_w", (D, dit["cond_dim"])), ("c_b", (D,))]
    elif dit["cond"] == COND_CLASS:
        out += [("table", (dit["cond_dim"] + 1, D))]
    for l in range(dit["depth"]):
        b = "blk%d." % l
        out += [(b + "ada_w", (6 * D, D)), (b + "ada_b", (6 * D,)),
                (b + "qkv_w", (3 * D, D)), (b + "qkv_b", (3 * D,)),
                (b + "proj_w", (D, D)), (b + "proj_b", (D,))]
        if dit["cond"] == COND_TEXT:
            out += [(b + "xq_w", (D, D)), (b + "xq_b", (D,)),
                    (b + "xkv_w", (2 * D, dit["cond_dim"])), (b + "xkv_b", (2 * D,)),
                    (b + "xo_w", (D, D)), (b + "xo_b", (D,))]
        out += [(b + "fc1_w", (R * D, D)), (b + "fc1_b", (R * D,)),
                (b + "fc2_w", (D, R * D)), (b + "fc2_b", (D,))]
    out += [("fin_ada_w", (2 * D, D)), ("fin_ada_b", (2 * D,)), ("fin_w", (P, D)), ("fin_b", (P,))]
    return out


def param_count(dit):
    return int(sum(int(np.prod(s)) for _, s in param_shapes(dit)))


def param_views(dit, flat):
    """dict name -> view of `flat` shaped as that tensor."""
    out, off = {}, 0
    for name, shape in param_shapes(dit):
        n = int(np.prod(shape))
        out[name] = flat[off:off + n].reshape(shape)
        off += n
    assert off == flat.size
    return out


def _rng(stream, cfg_idx):
    return np.random.Generator(np.random.Philox(key=BASE_SEED + stream + cfg_idx))


def weights(dit, cfg_idx=0, init="paper"):
    """Flat fp32 parameter array.
    init="paper": every scalar ~ N(0, 0.02) (the workload definition).
    init="loud":  test-only; Linear weights ~ N(0, 1/fan_in), biases ~ N(0, 0.25),
                  so that attention and MLP branches carry O(1) signal."""
    n = param_count(dit)
    rng = _rng(0, cfg_idx)
    flat = rng.standard_normal(n, dtype=np.float32)
    if init == "paper":
        flat *= np.float32(0.02)
        return flat
    assert init == "loud"
    for name, v in param_views(dit, flat).items():
        if name == "table":
            v *= np.float32(0.5)
        elif v.ndim == 2:
            v *= np.float32(1.0 / np.sqrt(v.shape[1]))
        else:
            v *= np.float32(0.5)
    return flat


def latent_noise(dit, batch, cfg_idx=0):
    """x_T ~ N(0, 1), [batch, in_ch, lat_h, lat_w] fp32."""
    return _rng(100, cfg_idx).standard_normal(
        (batch, dit["in_ch"], dit["lat_h"], dit["lat_w"]), dtype=np.float32)


def conditioning(dit, batch, cfg_idx=0, null=False):
    """Per-sample conditioning in the layout the library takes.
    vector: fp32 [batch, cond_dim] ~ N(0,1)        (null: zeros)
    class:  int32 [batch] uniform over classes     (null: the extra table row)
    text:   fp32 [batch, ctx_len, cond_dim] ~ N(0,1) (null: a second seeded draw)"""
    rng = _rng(300 if null else 200, cfg_idx)
    if dit["cond"] == COND_VECTOR:
        if null:
            return np.zeros((batch, dit["cond_dim"]), np.float32)
        return rng.standard_normal((batch, dit["cond_dim"]), dtype=np.float32)
    if dit["cond"] == COND_CLASS:
        if null:
            return np.full((batch,), dit["cond_dim"], np.int32)
        return rng.integers(0, dit["cond_dim"], size=(batch,), dtype=np.int32)
    return rng.standard_normal((batch, dit["ctx_len"], dit["cond_dim"]), dtype=np.float32)


def draft_pass(cfg_idx, taus):
    """Inputs of ONE full draft pass of configuration `cfg_idx` in the slot order the sampler uses,
    [draft i][cond | null][b]: seeded states x ~ N(0, 1) per slot (stream 400), the timestep taus[i]
    repeated over the g * batch slots of draft i, and the per-sample conditioning (null rows for the
    second half of every draft group when the configuration uses guidance).
    `taus` come from the caller's plan (one per draft); nothing is computed here.
    Returns (x [slots, C, H, W] fp32, t [slots] int32, cond [slots, ...])."""
    c = CONFIGS[cfg_idx]
    dit, B = c["dit"], c["batch"]
    g = 2 if c["guidance"] else 1
    m = len(taus)
    slots = m * g * B
    x = _rng(400, cfg_idx).standard_normal((slots, dit["in_ch"], dit["lat_h"], dit["lat_w"]), dtype=np.float32)
    t = np.repeat(np.asarray(taus, np.int32), g * B)
    rows = [conditioning(dit, B, cfg_idx)]
    if g == 2:
        rows.append(conditioning(dit, B, cfg_idx, null=True))
    cond = np.concatenate(rows * m, axis=0)
    return x, t, np.ascontiguousarray(cond)


def sample_points(count, size, tag):
    """`count` distinct flat indices into an array of `size` elements, seeded by `tag`: the
    positions at which stored reference values of large fields are kept."""
    rng = np.random.Generator(np.random.Philox(key=BASE_SEED + 900 + tag))
    return np.sort(rng.choice(size, size=min(count, size), replace=False))
