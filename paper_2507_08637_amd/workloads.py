"""Seeded synthetic workloads (the five benchmark configurations).

This module only draws random numbers and rounds them to the storage dtype; it
holds none of the method's arithmetic.  Both the CPU oracle's tests and the HIP
path's tests/bench take their inputs from here so that the two sides see the
same values.  The shapes follow the paper's ArXiv-128k experiment (Section 4:
128k tokens, small head dimension) and stand in for that dataset, which is not
available offline.

Arrays are returned as NumPy float32 whose values are exactly representable in
the configuration's storage dtype (bf16 values are rounded to nearest-even
once, here), so a float64 oracle and a bf16 kernel consume identical numbers.
"""
import numpy as np

CONFIGS = {
    1: dict(B=1, H=1, n=1024, d=64, L=3, m=64, dtype="f32", backward=False, flavour="plain"),
    2: dict(B=8, H=8, n=4096, d=64, L=4, m=128, dtype="bf16", backward=False, flavour="plain"),
    3: dict(B=4, H=12, n=16384, d=64, L=5, m=256, dtype="bf16", backward=True, flavour="spikes"),
    4: dict(B=1, H=8, n=131072, d=64, L=6, m=256, dtype="bf16", backward=True, flavour="sinusoid"),
    5: dict(B=2, H=16, n=65536, d=128, L=6, m=512, dtype="bf16", backward=True, flavour="plain"),
}

TENSOR_INDEX = dict(Q=0, K=1, V=2, Omega=3, Wg=4, bg=5, omega=6, dO=7, mask=8)


def round_to_bf16(x):
    """Round float32 array to the nearest bf16 (ties to even), keep float32 storage."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))
    out = ((bits + bias) & np.uint32(0xFFFF0000)).view(np.float32)
    return out


def _round(x, dtype):
    return round_to_bf16(x) if dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def make_inputs(B, H, n, d, L, m, dtype="f32", flavour="plain", seed_base=0, q_mean=0.0,
                zero_gate_w=False, backward=True, **_unused):
    """Draw one workload.  Returns a dict of float32 arrays plus scalars.

    flavour: "plain"    Q, K, V ~ N(0,1)
             "spikes"   as plain, then an independent Bernoulli(0.05) mask per entry
                        multiplies the entry by 10
             "sinusoid" as plain, then K[t, :] += sin(2 pi t / 4096)
             "smooth"   Q, K = 0.5 N(0,1) + 1.5 sin(2 pi t / 256), V = 0.3 N(0,1) + sin(2 pi t / 256):
                        a shared low-frequency component, so that the wavelet scales carry signal
             "smooth_cols" as smooth, but V = 0.3 N(0,1) + sin(2 pi t / 256) cos(x_j) + cos(2 pi t / 128) sin(x_j)
                        + 0.7 sin(2 pi t / 512) cos(2 x_j), x_j = 2 pi j / d: three column profiles with their own
                        time courses, so that the un-normalised output rows move in several directions
                        (a LayerNorm of rows that all share one profile has a vanishing Jacobian)
    q_mean shifts Q so that the pooled-query path carries signal.
    """
    def rng(name):
        return np.random.default_rng(seed_base + TENSOR_INDEX[name])

    shape = (B, H, n, d)
    out = {}
    for name in ("Q", "K", "V"):
        x = rng(name).standard_normal(shape, dtype=np.float32)
        if flavour == "spikes":
            # one mask stream per tensor, drawn after the tensor's own values
            mask = np.random.default_rng(seed_base + TENSOR_INDEX["mask"] + 10 * TENSOR_INDEX[name]
                                         ).random(shape, dtype=np.float32) < 0.05
            x = np.where(mask, x * np.float32(10.0), x)
        if flavour == "sinusoid" and name == "K":
            t = np.arange(n, dtype=np.float64)
            x = x + np.sin(2.0 * np.pi * t / 4096.0).astype(np.float32)[None, None, :, None]
        if flavour in ("smooth", "smooth_cols"):
            t = np.arange(n, dtype=np.float64)
            wave = np.sin(2.0 * np.pi * t / 256.0).astype(np.float32)[None, None, :, None]
            if flavour == "smooth_cols" and name == "V":
                xj = 2.0 * np.pi * np.arange(d) / d
                wave = (np.sin(2.0 * np.pi * t / 256.0)[:, None] * np.cos(xj)[None, :]
                        + np.cos(2.0 * np.pi * t / 128.0)[:, None] * np.sin(xj)[None, :]
                        + 0.7 * np.sin(2.0 * np.pi * t / 512.0)[:, None] * np.cos(2.0 * xj)[None, :]
                        ).astype(np.float32)[None, None, :, :]
            x = (np.float32(0.3) * x + wave) if name == "V" else (np.float32(0.5) * x + np.float32(1.5) * wave)
        if name == "Q" and q_mean != 0.0:
            x = x + np.float32(q_mean)
        out[name] = _round(x, dtype)
    out["Omega"] = _round(rng("Omega").standard_normal((d, m), dtype=np.float32), dtype)
    if zero_gate_w:
        out["Wg"] = np.zeros((H, L + 1, d), dtype=np.float32)
    else:
        out["Wg"] = rng("Wg").standard_normal((H, L + 1, d), dtype=np.float32)
    out["bg"] = (0.1 * rng("bg").standard_normal((H, L + 1))).astype(np.float32)
    if zero_gate_w:
        out["omega"] = np.ones(L + 1, dtype=np.float32)
    else:
        out["omega"] = (1.0 + 0.1 * rng("omega").standard_normal(L + 1)).astype(np.float32)
    out["sigma"] = np.float32(1.0)
    if backward:
        out["dO"] = _round(rng("dO").standard_normal(shape, dtype=np.float32), dtype)
    return out


BLOCK_TENSOR_INDEX = dict(X=0, WQ=10, WK=11, WV=12, WO=13, dY=7)


def make_block_inputs(B, H, n, d, L, m, seed_base=0, x_mean=0.0, backward=True, **_unused):
    """Inputs of the attention block (bf16 storage): X (B, n, H*d) ~ N(0,1) + x_mean, the four
    hidden x hidden weights ~ N(0, 1/hidden), dY ~ N(0,1); the core's parameters as in make_inputs."""
    hidden = H * d

    def rng(name):
        return np.random.default_rng(seed_base + BLOCK_TENSOR_INDEX[name])

    out = {}
    x = rng("X").standard_normal((B, n, hidden), dtype=np.float32)
    if x_mean != 0.0:
        x += np.float32(x_mean)
    out["X"] = round_to_bf16(x)
    for name in ("WQ", "WK", "WV", "WO"):
        w = rng(name).standard_normal((hidden, hidden), dtype=np.float32) / np.float32(np.sqrt(hidden))
        out[name] = round_to_bf16(w)
    core = make_inputs(1, H, 1, d, L, m, dtype="bf16", seed_base=seed_base, backward=False)
    for name in ("Omega", "Wg", "bg", "omega", "sigma"):
        out[name] = core[name]
    if backward:
        out["dY"] = round_to_bf16(rng("dY").standard_normal((B, n, hidden), dtype=np.float32))
    return out


def make_config(idx, **override):
    """Inputs for benchmark configuration idx (1..5); seed = 1000 * idx + tensor index."""
    cfg = dict(CONFIGS[idx])
    cfg.update(override)
    cfg.setdefault("seed_base", 1000 * idx)
    if idx == 1:
        cfg.setdefault("zero_gate_w", True)   # gate logits supplied directly through the bias
    return cfg, make_inputs(**cfg)
