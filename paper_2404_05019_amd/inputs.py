"""Seeded synthetic inputs for one ScMoE layer.

This module only draws random numbers and formats them; it holds none of the layer's
arithmetic, so the CPU oracle and the GPU library can both be fed from it.  The workloads
stand in for the SwinV2-MoE-S stage-3 and GPT-style layers of the paper's Tables 8-9,
whose real activations would need trained checkpoints: activations ~ N(0,1), weights
~ N(0, 0.02), drawn in fp32 and rounded once (ties to even) to the layer's storage type.
"""
import numpy as np

# name -> shape of the layer.  `cf` is the capacity factor; C = ceil(cf*k*T/E).
CONFIGS = {
    "tiny":   dict(T=256,   d=64,   F=256,  E=4,  k=1, cf=1.25, dtype="f32",  seed=0, zipf=None),
    "small":  dict(T=8192,  d=384,  F=1536, E=8,  k=1, cf=1.25, dtype="bf16", seed=1, zipf=None),
    "medium": dict(T=16384, d=1024, F=4096, E=8,  k=1, cf=1.25, dtype="bf16", seed=2, zipf=None),
    "skewed": dict(T=16384, d=1024, F=4096, E=16, k=1, cf=1.0,  dtype="bf16", seed=3, zipf=1.2),
    "large":  dict(T=32768, d=2048, F=8192, E=16, k=1, cf=1.25, dtype="bf16", seed=4, zipf=None),
}


def capacity(T, E, k, cf):
    """ceil(cf*k*T/E) in exact rational arithmetic (cf given to at most 6 decimals)."""
    num = int(round(cf * 1_000_000)) * k * T
    den = 1_000_000 * E
    return -(-num // den)


def bf16_bits(a):
    """Round float32 -> bf16 (ties to even).  Returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_widen(bits):
    """uint16 bf16 bit patterns -> the same values as float32."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(a, dtype):
    """Values of `a` after storage in `dtype`, as float32 (identity for f32)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_widen(bf16_bits(a))
    return a


def _normal(rng, shape, scale, dtype):
    a = rng.standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        a *= np.float32(scale)
    return quantize(a, dtype)


def zipf_bias(col_sigma, s, seed, n_mc=400_000, iters=60):
    """Per-expert additive gate bias that makes the expected top-1 load Zipf(s).

    Model: logit_e ~ N(0, col_sigma[e]^2), independent (x ~ N(0,1) rows against the
    columns of W_g).  On a fixed Monte-Carlo sample of such logits the bias is iterated,
    bias_e += 0.7 * sigma * ln(q_e / load_e), until the arg-max frequencies match
    q_e ~ (e+1)^-s.  Only the distribution of the data is shaped here; the layer's own
    gate is not evaluated.
    """
    E = len(col_sigma)
    q = (np.arange(1, E + 1, dtype=np.float64)) ** (-float(s))
    q /= q.sum()
    rng = np.random.default_rng(seed + 7919)
    z = rng.standard_normal((n_mc, E)) * np.asarray(col_sigma, np.float64)[None, :]
    sig = float(np.mean(col_sigma))
    b = sig * np.log(q)
    for _ in range(iters):
        load = np.bincount(np.argmax(z + b[None, :], axis=1), minlength=E) / n_mc
        load = np.maximum(load, 1e-6)
        b += 0.7 * sig * np.log(q / load)
        b -= b.max()
    return b.astype(np.float32)


def make_layer(T, d, F, E, dtype="bf16", seed=0, zipf=None, biases=False, cg_rows=0,
               w_scale=0.02, x_scale=1.0, **_unused):
    """Draw all tensors of one layer.  Returns a dict of float32 numpy arrays whose values
    are exactly representable in `dtype` (gate matrix, gate bias, FFN biases and the
    coefficient-gate matrix stay fp32).

    keys: x_prev, x_cur [T,d]; Wg [d,E]; bias [E] or None; W1 [E,F,d]; W2 [E,d,F];
    W1s [F,d]; W2s [d,F]; b1,b2,b1s,b2s (None unless biases); Wcg [cg_rows,d] or None.
    """
    rng = np.random.default_rng(seed)
    L = {}
    L["x_prev"] = _normal(rng, (T, d), x_scale, dtype)
    L["x_cur"] = _normal(rng, (T, d), x_scale, dtype)
    L["Wg"] = _normal(rng, (d, E), w_scale, "f32")
    L["W1"] = _normal(rng, (E, F, d), w_scale, dtype)
    L["W2"] = _normal(rng, (E, d, F), w_scale, dtype)
    L["W1s"] = _normal(rng, (F, d), w_scale, dtype)
    L["W2s"] = _normal(rng, (d, F), w_scale, dtype)
    if biases:
        L["b1"] = _normal(rng, (E, F), w_scale, "f32")
        L["b2"] = _normal(rng, (E, d), w_scale, "f32")
        L["b1s"] = _normal(rng, (F,), w_scale, "f32")
        L["b2s"] = _normal(rng, (d,), w_scale, "f32")
    else:
        L["b1"] = L["b2"] = L["b1s"] = L["b2s"] = None
    L["Wcg"] = _normal(rng, (cg_rows, d), w_scale, "f32") if cg_rows else None
    if zipf is not None:
        col_sigma = np.sqrt((L["Wg"].astype(np.float64) ** 2).sum(axis=0)) * x_scale
        L["bias"] = zipf_bias(col_sigma, zipf, seed)
    else:
        L["bias"] = None
    return L


def make_config(name, **overrides):
    """Tensors of a named configuration plus its shape dict (with capacity `C`)."""
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    cfg["C"] = capacity(cfg["T"], cfg["E"], cfg["k"], cfg["cf"])
    return make_layer(**cfg), cfg
