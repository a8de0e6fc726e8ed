"""Parity of the HIP path (through the C-ABI) against the float64 oracle on seeded inputs.

Tolerances (relative Frobenius error per output tensor): 1e-4 for float32, 2e-2 for bf16.
bf16 inputs are rounded once on the host; the oracle consumes those rounded values in float64.
"""
import numpy as np
import pytest

from paper_2507_08637_amd import workloads
from tests import helpers as hp

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
# MFMA path, gate-parameter gradients on random inputs: absolute error allowed as a fraction of the
# un-cancelled magnitude of the sum (see _check_mfma); strict 2e-2 relative error is required
# where the gradient carries signal (test_mfma_gate_gradients_with_signal).
GATE_NOISE_TOL = 5e-2


def _check_all(res, ref, tol, names=("O", "dQ", "dK", "dV", "dWg", "dbg", "domega"), where=""):
    errs = {k: hp.rel_err(res[k], ref[k]) for k in names}
    print(where, {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    bad = {k: v for k, v in errs.items() if not v < tol}
    assert not bad, (where, bad)
    return errs


def _check_mfma(res, ref, p, cfg, where="", noise_limited=False, eps=1e-6, pooled=False, layernorm=False):
    """MFMA path against the plain float64 oracle.  O, dQ, dK, dV: 2e-2 relative Frobenius error,
    always.  Gate-parameter gradients (dW_g, db_g, d omega): the same plain 2e-2, unless the case
    is listed as noise-limited: these gradients are inner products of dX_F (a tensor that itself
    carries the 2e-2 tolerance) with the wavelet bands of X, and on small seeded random inputs they
    cancel down to their statistical noise floor, where a relative error says nothing.  For those
    listed cases the error is bounded against the un-cancelled magnitude of the sum
    (helpers.gate_grad_scales), both sides taking the ReLU decision at the kernel's precision
    (X_F rounded to fp16 before the projection); the plain relative error is printed.  Every kernel
    variant that has such a case also has a signal-carrying case held to the plain 2e-2
    (test_mfma_gate_gradients_with_signal)."""
    _check_all(res, ref, 2e-2, names=("O", "dQ", "dK", "dV"), where=where)
    plain = {k: hp.rel_err(res[k], ref[k]) for k in ("dWg", "dbg", "domega")}
    strict_ok = all(v < 2e-2 for v in plain.values())
    print(where, "gate grads, plain relative", {k: f"{v:.2e}" for k, v in plain.items()},
          "STRICT-OK" if strict_ok else "ABOVE-2e-2", flush=True)
    if not noise_limited:
        assert strict_ok, (where, plain)
        return
    scales = hp.gate_grad_scales(p, cfg, eps=eps, layernorm=layernorm)
    ref16 = hp.oracle_backward(p, cfg, eps=eps, proj_dtype=np.float16, pooled=pooled, layernorm=layernorm)
    errs = {k: hp.scaled_err(res[k], ref16[k], scales[k]) for k in ("dWg", "dbg", "domega")}
    print(where, "gate grads vs un-cancelled scale", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    bad = {k: v for k, v in errs.items() if not v < GATE_NOISE_TOL}
    assert not bad, (where, bad)


SMALL = [
    # multi-tile, ragged tail in n (200 = 3 tiles + 8 rows), d and m not multiples of 64
    dict(B=2, H=3, n=200, d=48, L=3, m=80),
    dict(B=1, H=2, n=512, d=64, L=6, m=128),
    dict(B=2, H=2, n=320, d=128, L=5, m=256),
    dict(B=1, H=1, n=64, d=64, L=6, m=64),      # a single Haar block
    dict(B=1, H=2, n=16, d=16, L=4, m=16),      # smallest sizes
    dict(B=1, H=2, n=96, d=32, L=0, m=32),      # no wavelet levels: F has one entry
    dict(B=3, H=1, n=256, d=256, L=2, m=48),    # maximum head dim
    dict(B=2, H=2, n=203, d=32, L=3, m=48),     # n not a multiple of 2^L: zero padding of Algorithm 2 in-kernel
    dict(B=1, H=2, n=100, d=64, L=6, m=64),     # n between 2^L and 2^(L+1)
    dict(B=1, H=1, n=5, d=16, L=2, m=16),       # n barely above one block
    dict(B=2, H=1, n=1, d=16, L=3, m=16),       # a single token: the block is all padding but one row
    # transforms deeper than one 64-row tile: two and three stages, ragged tiles at every stage
    dict(B=1, H=2, n=1000, d=32, L=8, m=32),    # blocks of 256 rows: 16 tiles, then 4 blocks of 4 tile coefficients
    dict(B=2, H=1, n=4177, d=48, L=12, m=32),   # 66 tiles -> 2 tiles at the second stage, one block of 4096 rows + tail
    # three stages (6 + 6 + 1): 8192-row block larger than n.  (Own seed: with the common one this
    # shape has a pre-activation within float32 rounding of zero, its ReLU derivative flips against
    # float64 and that single element puts dK at 5e-3; every other output agrees to 1e-6.)
    dict(B=1, H=1, n=4500, d=16, L=13, m=16, seed=77),
    dict(B=1, H=1, n=300, d=16, L=7, m=16),     # last stage with one level on 5 coefficients
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SMALL, ids=lambda s: "B{B}H{H}n{n}d{d}L{L}m{m}".format(**s))
def test_small_shapes_forward_backward(shape, dtype):
    shape = dict(shape)
    cfg = dict(shape, dtype=dtype, flavour="plain", seed_base=shape.pop("seed", 4242), q_mean=0.5)
    cfg.pop("seed", None)
    p = workloads.make_inputs(**cfg)
    res = hp.gpu_forward_backward(p, cfg, flags=1)   # generic path for every shape and dtype
    ref = hp.oracle_backward(p, cfg)
    names = ("O", "dQ", "dK", "dV", "dWg", "dbg", "domega")
    if shape["L"] == 0:
        # One band only: X_F = F_0 X, and a common scale of Q_F, K_F cancels in O up to eps
        # (ReLU is positively homogeneous), so dF_0 is an eps-order remainder of a cancelling sum.
        # Its relative error means nothing; require it to be tiny against the un-cancelled scale.
        names = ("O", "dQ", "dK", "dV")
        scale = float(np.linalg.norm(ref["dQ"]) * np.linalg.norm(p["Q"]))
        assert float(res["domega"].abs().max().cpu()) < 1e-3 * scale
    if shape["n"] == 1:
        # One token: O = V whatever Q and K are (numerator and normaliser carry the same single
        # feature product), so every gradient but dV is an eps-order remainder of terms that
        # cancel.  Require those to be tiny against dV instead of comparing noise with noise.
        names = ("O", "dV")
        scale = float(np.linalg.norm(ref["dV"]))
        for k in ("dQ", "dK", "dWg", "dbg", "domega"):
            assert float(res[k].float().norm().cpu()) < 1e-3 * scale, k
            assert float(np.linalg.norm(ref[k])) < 1e-3 * scale, k
    _check_all(res, ref, TOL[dtype], names=names, where=f"{shape} {dtype}")


# noise=True: seeded random inputs on which the gate-parameter gradients sit at their noise floor
# (measured plain relative errors of dW_g / d omega in the comment; see _check_mfma)
MFMA_SHAPES = [
    dict(B=1, H=1, n=64, d=64, L=6, m=128, noise=True),       # one Haar block, one wave active  (1.4e-2 / 3.0e-2)
    dict(B=2, H=2, n=320, d=64, L=6, m=256),      # 5 blocks: last workgroup partly idle
    dict(B=1, H=3, n=1024, d=64, L=3, m=384),     # three feature blocks of 128
    dict(B=1, H=2, n=704, d=64, L=0, m=128, noise=True),      # no wavelet levels (dF_0 is an eps-order remainder)
    dict(B=1, H=2, n=640, d=64, L=0, m=256, noise=True),      # no wavelet levels, 256 features per pass
    dict(B=2, H=1, n=4096, d=64, L=5, m=512, noise=True),     # two operand chunks in the rows kernel  (9.8e-3 / 6.0e-2)
    dict(B=1, H=2, n=2560, d=64, L=1, m=256, noise=True),     # (1.3e-2 / 2.3e-2)
    dict(B=1, H=1, n=64, d=128, L=6, m=128, noise=True),      # head dimension 128  (3.3e-3 / 2.6e-2)
    dict(B=2, H=2, n=832, d=128, L=6, m=512),     # 13 blocks, four operand chunks
    dict(B=1, H=2, n=1536, d=128, L=4, m=256),
    dict(B=1, H=1, n=256, d=64, L=4, m=4096, noise=True),     # maximum feature count: 16 operand chunks per row group  (7.0e-2 / 1.2e-1)
    dict(B=6, H=8, n=128, d=64, L=5, m=128),      # 48 slices of two blocks: more workgroups than row groups
    dict(B=33, H=31, n=64, d=64, L=4, m=128),     # 1023 slices, the most the library takes
    # sequence lengths that are not multiples of the 64-row block: the last block is partial
    dict(B=2, H=2, n=1000, d=64, L=6, m=256),     # 15 full blocks + 40 rows
    dict(B=1, H=2, n=100, d=64, L=5, m=128),      # one full block + 36 rows
    dict(B=1, H=1, n=40, d=64, L=3, m=128, noise=True),       # less than one block  (2.2e-1 / 6.0e-1)
    dict(B=1, H=2, n=203, d=128, L=6, m=128, noise=True),     # head dimension 128, 3 blocks + 11 rows  (1.2e-2 / 4.6e-2)
]


@pytest.mark.parametrize("shape", MFMA_SHAPES, ids=lambda s: "B{B}H{H}n{n}d{d}L{L}m{m}".format(**s))
def test_mfma_path_shapes(shape):
    """bf16 shapes that run on the MFMA path (checked through wersa_selected_path)."""
    import torch
    from paper_2507_08637_amd import binding
    shape = dict(shape)
    noise = shape.pop("noise", False)
    cfg = dict(shape, dtype="bf16", flavour="plain", seed_base=555, q_mean=0.5)
    probe = torch.empty(cfg["B"], cfg["H"], cfg["n"], cfg["d"], dtype=torch.bfloat16, device="cuda")
    assert binding.wersa_path_name(binding.make_desc(probe, cfg["L"], cfg["m"])) == "mfma"
    p = workloads.make_inputs(**cfg)
    res = hp.gpu_forward_backward(p, cfg)
    ref = hp.oracle_backward(p, cfg)
    _check_mfma(res, ref, p, cfg, where=f"mfma {shape}", noise_limited=noise)
    fwd = hp.oracle_forward(p, cfg)
    sl = cfg["B"] * cfg["H"]
    for name in ("qbar", "s", "F", "S", "z", "D"):
        r = fwd[name].reshape((sl,) + fwd[name].shape[2:])
        e = hp.rel_err(res["saved"][name], r)
        assert e < 2e-2, (name, e)


def _signal_problem(cfg, eps=1e-6, pooled=False, layernorm=False, separate_omega=False):
    """A workload on which the gate-parameter gradients are coherent sums: Q, K, V share a
    low-frequency component and the loss is 0.5 ||O - T||^2 with a phase-shifted target T, so that
    dO = O - T (O from the oracle's forward).  With the LayerNorm output stage the loss is the
    linear one <O, T> with a target that also varies over the columns, dO = T: a normalised row
    has a fixed norm and is orthogonal to anything constant along the row, so the quadratic loss
    would leave a gradient that is the small difference of nearly equal terms, dominated by the
    rounding of O."""
    p = workloads.make_inputs(**cfg)
    if separate_omega:
        omk = np.random.default_rng(3199).standard_normal(p["Omega"].shape, dtype=np.float32)
        p["OmegaK"] = workloads.round_to_bf16(omk)
    if pooled:
        from oracle import wersa_oracle as wo
        O = wo.forward(p["Q"], p["K"], p["V"], p["Omega"], float(p["sigma"]), p["Wg"], p["bg"], p["omega"],
                       cfg["L"], eps=eps, pooled=True, keep=("O",))["O"]
    else:
        O = hp.oracle_forward(p, cfg, eps=eps, keep=("O",), layernorm=layernorm)["O"]
    t = np.arange(cfg["n"])
    T = np.cos(2 * np.pi * t / 256.0)[None, None, :, None]
    if layernorm:
        xj = 2 * np.pi * np.arange(cfg["d"]) / cfg["d"]
        T = (np.sin(2 * np.pi * t / 256.0)[:, None] * np.sin(xj + 0.7)[None, :]
             + 0.5 * np.cos(2 * np.pi * t / 128.0)[:, None] * np.cos(2 * xj + 0.3)[None, :])[None, None]
        p["dO"] = workloads.round_to_bf16(np.broadcast_to(T, O.shape).astype(np.float32))
    else:
        p["dO"] = workloads.round_to_bf16((O - T).astype(np.float32))
    return p


SIGNAL_CASES = {
    # one per kernel variant of the MFMA path (all at the plain 2e-2 on every output)
    "d64_m256_dv_inside": (dict(B=1, H=2, n=2048, d=64, L=4, m=256), {}),
    "d64_m128": (dict(B=1, H=2, n=2048, d=64, L=5, m=128), {}),
    "d64_m512_two_chunks": (dict(B=1, H=2, n=2048, d=64, L=5, m=512), {}),
    "d64_one_level": (dict(B=1, H=2, n=2560, d=64, L=1, m=256), {}),
    "d128": (dict(B=1, H=2, n=2048, d=128, L=5, m=256), {}),
    "d128_m512": (dict(B=1, H=2, n=2048, d=128, L=6, m=512), {}),
    "ragged": (dict(B=1, H=2, n=2000, d=64, L=6, m=256), {}),
    "ragged_d128": (dict(B=1, H=2, n=1992, d=128, L=6, m=128), {}),
    "deep": (dict(B=1, H=2, n=4096, d=64, L=9, m=256), {}),
    "deep_d128": (dict(B=1, H=2, n=4096, d=128, L=8, m=128), {}),
    "deep_ragged": (dict(B=1, H=2, n=4000, d=64, L=8, m=256), {}),
    # (min_signal: with the LayerNorm output stage, and with unrelated feature maps for Q and K, the
    # shared component gives a smaller coherent part: about 2 x and 0.5 x the un-cancelled scale)
    "layernorm": (dict(B=1, H=2, n=2048, d=64, L=4, m=256, flavour="smooth_cols"),
                  dict(flags=8, eps=1e-3, layernorm=True, min_signal=1.0)),
    "pooled_gate": (dict(B=2, H=3, n=2048, d=64, L=4, m=256), dict(flags=4, pooled=True)),
    "separate_omega": (dict(B=1, H=2, n=2048, d=64, L=4, m=256), dict(flags=2, separate_omega=True, min_signal=0.3)),
}


@pytest.mark.parametrize("case", sorted(SIGNAL_CASES))
def test_mfma_gate_gradients_with_signal(case):
    """Gate-parameter gradients at the plain tolerance on every kernel variant of the MFMA path,
    on workloads where they are well above the noise floor (see _signal_problem)."""
    shape, kw = SIGNAL_CASES[case]
    flags, eps = kw.get("flags", 0), kw.get("eps", 1e-6)
    pooled, layernorm = kw.get("pooled", False), kw.get("layernorm", False)
    cfg = dict(dict(flavour="smooth"), **shape, dtype="bf16", seed_base=777)
    p = _signal_problem(cfg, eps=eps, pooled=pooled, layernorm=layernorm, separate_omega=kw.get("separate_omega", False))
    res = hp.gpu_forward_backward(p, cfg, flags=flags, eps=eps)
    ref = hp.oracle_backward(p, cfg, eps=eps, pooled=pooled, layernorm=layernorm)
    scales = hp.gate_grad_scales(p, cfg, eps=eps, layernorm=layernorm)   # (per-head gates: the same order when pooled)
    signal = float(np.linalg.norm(ref["domega"]) / np.linalg.norm(scales["domega"]))
    # the premise of this test: |dF| well above the error a 2e-2 tensor can leave in a cancelling sum
    assert signal > kw.get("min_signal", 3.0), signal
    _check_all(res, ref, 2e-2, where=f"mfma, gate gradients with signal: {case} (x{signal:.0f} the noise scale)")


@pytest.mark.parametrize("d", [64, 128])
def test_mfma_dsigma_against_the_oracle(d):
    """d sigma of the default normaliser on the MFMA path (Section 3.1 step 7's bandwidth reaches
    the output only through eps, so eps = 1e-2 makes the gradient measurable): the kernels' closed
    form (2 eps / sigma) sum_t dD_t against the oracle's term-by-term chain rule, on a workload
    where the sum is coherent; and zero below the bandwidth floor."""
    eps = 1e-2
    cfg = dict(B=1, H=2, n=2048, d=d, L=4, m=256, dtype="bf16", flavour="smooth", seed_base=777)
    p = _signal_problem(cfg, eps=eps)
    p["sigma"] = np.float32(1.5)
    p = dict(p)
    res = hp.gpu_forward_backward(p, cfg, eps=eps)
    ref = hp.oracle_backward(p, cfg, eps=eps)
    _check_all(res, ref, 2e-2, where=f"mfma d sigma, d={d}")
    got = float(res["dsigma"].cpu()[0])
    print(f"d sigma d={d}: gpu {got:.6e} oracle {ref['dsigma']:.6e}", flush=True)
    assert abs(ref["dsigma"]) > 1e-3                                    # the premise: measurable
    assert abs(got - ref["dsigma"]) < 2e-2 * abs(ref["dsigma"]), (got, ref["dsigma"])
    res2 = hp.gpu_forward_backward(p, cfg, eps=eps, bw_floor=2.0)
    ref2 = hp.oracle_backward(p, cfg, eps=eps, bw_floor=2.0)
    assert float(res2["dsigma"].cpu()[0]) == 0.0 and ref2["dsigma"] == 0.0
    _check_all(res2, ref2, 2e-2, names=("O", "dQ", "dK", "dV"), where="mfma, sigma below the floor")


@pytest.mark.parametrize("case", ["large", "tiny", "large_scale_weights", "mixed"])
def test_mfma_path_input_range(case):
    """The MFMA path rounds X_F to fp16 before the projection (Section 3.1 step 7).  ReLU is
    positively homogeneous, so a power of two chosen per slice from max|Q| and the filter keeps
    those operands in range: inputs (and the bandwidth with them) of the order 2^13 or 2^-20, and
    per-scale weights of the order 2^10, must meet the same bar as inputs of order one.  (Without
    the scale, 2^13 inputs overflow fp16 to infinity and 2^-20 inputs vanish below its subnormals.)
    'mixed': K sixteen times larger than Q."""
    import torch
    from paper_2507_08637_amd import binding
    cfg = dict(B=1, H=2, n=1024, d=64, L=5, m=256, dtype="bf16", flavour="plain", seed_base=8800, q_mean=0.3)
    p = workloads.make_inputs(**cfg)
    f = {"large": 2.0 ** 13, "tiny": 2.0 ** -20, "large_scale_weights": 1.0, "mixed": 1.0}[case]
    for k in ("Q", "K"):
        p[k] = (p[k] * np.float32(f)).astype(np.float32)     # exact: a power of two
    p["sigma"] = np.float32(f)
    p["Wg"] = (p["Wg"] / np.float32(f)).astype(np.float32)   # the gate's logits stay of order one
    if case == "large_scale_weights":
        p["omega"] = (p["omega"] * np.float32(1024.0)).astype(np.float32)
    if case == "mixed":
        p["K"] = (p["K"] * np.float32(16.0)).astype(np.float32)
    probe = torch.empty(cfg["B"], cfg["H"], cfg["n"], cfg["d"], dtype=torch.bfloat16, device="cuda")
    assert binding.wersa_path_name(binding.make_desc(probe, cfg["L"], cfg["m"])) == "mfma"
    res = hp.gpu_forward_backward(p, cfg)
    for k in ("O", "dQ", "dK", "dV", "dWg", "dbg", "domega"):
        assert bool(torch.isfinite(res[k].float()).all()), k
    ref = hp.oracle_backward(p, cfg)
    _check_all(res, ref, 2e-2, names=("O", "dQ", "dK", "dV"), where=f"mfma input range: {case}")
    fwd = hp.oracle_forward(p, cfg)
    sl = cfg["B"] * cfg["H"]
    for name in ("S", "z", "D"):
        r = fwd[name].reshape((sl,) + fwd[name].shape[2:])
        assert hp.rel_err(res["saved"][name], r) < 2e-2, name
    _check_mfma(res, ref, p, cfg, where=f"mfma input range: {case}")   # plain 1.3e-2 .. 1.5e-2, as at order one
    if case == "large":
        # The factor is a power of two, so against the run on the unscaled inputs the outputs must carry
        # exact powers of it: O, dV, d b_g, d omega none, dQ and dK 1/f, d W_g f (W_g was divided by f).
        base = hp.gpu_forward_backward(workloads.make_inputs(**cfg), cfg)
        for k, e in dict(O=0, dV=0, dQ=-1, dK=-1, dWg=1, dbg=0, domega=0).items():
            assert torch.equal(res[k].double() / f ** e, base[k].double()), k


def test_mfma_and_generic_paths_agree():
    """Same bf16 problem through both paths (descriptor flag): both within tolerance of the
    oracle, hence of each other."""
    cfg = dict(B=1, H=2, n=1024, d=64, L=4, m=256, dtype="bf16", flavour="spikes", seed_base=31, q_mean=0.3)
    p = workloads.make_inputs(**cfg)
    ref = hp.oracle_backward(p, cfg)
    from paper_2507_08637_amd import binding
    res = hp.gpu_forward_backward(p, cfg, flags=binding.WERSA_FLAG_GENERIC_PATH)
    _check_all(res, ref, 2e-2, where="generic path")
    res = hp.gpu_forward_backward(p, cfg, flags=0)
    _check_mfma(res, ref, p, cfg, where="mfma path")


def test_mfma_strided_layout():
    cfg = dict(B=2, H=2, n=256, d=64, L=4, m=128, dtype="bf16", flavour="plain", seed_base=8, q_mean=0.5)
    p = workloads.make_inputs(**cfg)
    res = hp.gpu_forward_backward(p, cfg, layout="bnhd")
    ref = hp.oracle_backward(p, cfg)
    _check_mfma(res, ref, p, cfg, where="mfma strided", noise_limited=True)   # n = 256, random: plain 2.0e-2 on db_g


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_saved_stage_tensors(dtype):
    """q-bar, gate, F, S, z and the normaliser D (steps 4, 7, 8) against the oracle's stages."""
    cfg = dict(B=2, H=2, n=384, d=64, L=4, m=96, dtype=dtype, flavour="plain", seed_base=99, q_mean=0.3)
    p = workloads.make_inputs(**cfg)
    res = hp.gpu_forward_backward(p, cfg, backward=False)
    ref = hp.oracle_forward(p, cfg)
    sl = cfg["B"] * cfg["H"]
    for name in ("qbar", "s", "F", "S", "z", "D"):
        r = ref[name].reshape((sl,) + ref[name].shape[2:])
        e = hp.rel_err(res["saved"][name], r)
        assert e < TOL[dtype], (name, e)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_strided_layout(dtype):
    """Heads addressed by stride: tensors stored (B, n, H, d), presented as (B, H, n, d)."""
    cfg = dict(B=2, H=3, n=128, d=32, L=3, m=64, dtype=dtype, flavour="plain", seed_base=7, q_mean=0.5)
    p = workloads.make_inputs(**cfg)
    res = hp.gpu_forward_backward(p, cfg, layout="bnhd")
    ref = hp.oracle_backward(p, cfg)
    _check_all(res, ref, TOL[dtype], where="strided")


def test_dsigma_closed_form_and_floor():
    """sigma reaches the output only through eps; with a large eps the gradient is measurable.
    Compared with the oracle's term-by-term chain rule, relative to 2 eps/sigma * sum|dD|."""
    eps = 1e-2
    cfg = dict(B=2, H=2, n=256, d=32, L=3, m=64, dtype="f32", flavour="plain", seed_base=11, q_mean=0.5)
    p = workloads.make_inputs(**cfg)
    p["sigma"] = np.float32(1.5)
    res = hp.gpu_forward_backward(p, cfg, eps=eps)
    ref = hp.oracle_backward(p, cfg, eps=eps)
    _check_all(res, ref, 1e-4, where="eps=1e-2")
    got = float(res["dsigma"].cpu()[0])
    assert abs(got - ref["dsigma"]) < 1e-3 * abs(ref["dsigma"]) + 1e-7, (got, ref["dsigma"])
    # below the floor the bandwidth is clamped and receives no gradient
    res2 = hp.gpu_forward_backward(p, cfg, eps=eps, bw_floor=2.0)
    ref2 = hp.oracle_backward(p, cfg, eps=eps, bw_floor=2.0)
    assert float(res2["dsigma"].cpu()[0]) == 0.0 and ref2["dsigma"] == 0.0
    _check_all(res2, ref2, 1e-4, names=("O", "dQ"), where="floor")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_haar_filter_stage(dtype):
    """The gated Haar stage alone (steps 3, 5, 6) against the oracle's lifting recursion."""
    import torch
    from oracle import wersa_oracle as wo
    from paper_2507_08637_amd import binding
    B, H, n, d, L = 2, 2, 448, 80, 6
    rng = np.random.default_rng(5)
    x = rng.standard_normal((B, H, n, d)).astype(np.float32)
    if dtype == "bf16":
        x = workloads.round_to_bf16(x)
    filt = rng.uniform(0.0, 1.5, (B * H, L + 1)).astype(np.float32)
    xt = torch.from_numpy(x).cuda().to(torch.float32 if dtype == "f32" else torch.bfloat16)
    y = binding.wersa_haar_filter(xt, torch.from_numpy(filt).cuda(), L)
    torch.cuda.synchronize()
    ref = np.stack([wo.haar_filter(x[b, h].astype(np.float64), filt[b * H + h].astype(np.float64), L)
                    for b in range(B) for h in range(H)]).reshape(B, H, n, d)
    tol = 1e-6 if dtype == "f32" else 4e-3   # bf16 output rounding: 2^-9 per element
    assert hp.rel_err(y, ref) < tol
    # all-ones filter reproduces the input exactly up to float32 rounding of the lifting steps
    y1 = binding.wersa_haar_filter(xt, torch.ones(B * H, L + 1, device="cuda"), L)
    assert hp.rel_err(y1, x.astype(np.float64)) < tol


@pytest.mark.parametrize("shape", [dict(B=1, H=2, n=203, d=48, L=3),      # partial last tile, partial column tile
                                   dict(B=2, H=2, n=1000, d=128, L=6),    # two column tiles
                                   dict(B=1, H=3, n=64, d=16, L=0),       # no levels: a plain scale by F_0
                                   dict(B=2, H=2, n=640, d=64, L=5, layout="bnhd")])   # heads addressed by stride
def test_haar_filter_stage_bf16_streaming_kernel(shape):
    """The stage entry point on bf16 tensors (one streaming kernel in block-mean form, 16-byte row
    pieces) against the oracle's lifting recursion, edge shapes; the float32-arithmetic kernel
    behind WERSA_FLAG_GENERIC_PATH must agree with it to the output rounding."""
    import torch
    from oracle import wersa_oracle as wo
    from paper_2507_08637_amd import binding
    B, H, n, d, L = (shape[k] for k in ("B", "H", "n", "d", "L"))
    rng = np.random.default_rng(9)
    x = workloads.round_to_bf16((rng.standard_normal((B, H, n, d)) + 0.2).astype(np.float32))
    filt = rng.uniform(-0.5, 1.5, (B * H, L + 1)).astype(np.float32)
    xt = torch.from_numpy(x).cuda().to(torch.bfloat16)
    if shape.get("layout") == "bnhd":
        xt = xt.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    y = torch.full_like(xt, float("nan"))
    binding.wersa_haar_filter(xt, torch.from_numpy(filt).cuda(), L, out=y)
    torch.cuda.synchronize()
    ref = np.stack([wo.haar_filter(x[b, h].astype(np.float64), filt[b * H + h].astype(np.float64), L)
                    for b in range(B) for h in range(H)]).reshape(B, H, n, d)
    assert bool(torch.isfinite(y.float()).all())
    assert hp.rel_err(y, ref) < 4e-3   # bf16 output rounding: 2^-9 per element


@pytest.mark.parametrize("shape", [dict(n=4160, L=12), dict(n=1000, L=9), dict(n=5000, L=7)])
def test_haar_filter_stage_deeper_than_one_tile(shape):
    """The stage entry point with a workspace: levels above 6 run on the approximation
    coefficients of the tiles (sequence lengths with a partial last tile and a partial last
    block included)."""
    import torch
    from oracle import wersa_oracle as wo
    from paper_2507_08637_amd import binding
    B, H, d = 1, 2, 48
    n, L = shape["n"], shape["L"]
    rng = np.random.default_rng(7)
    x = (rng.standard_normal((B, H, n, d)) + 0.3).astype(np.float32)
    filt = rng.uniform(0.0, 1.5, (B * H, L + 1)).astype(np.float32)
    xt = torch.from_numpy(x).cuda()
    y = binding.wersa_haar_filter(xt, torch.from_numpy(filt).cuda(), L)
    torch.cuda.synchronize()
    ref = np.stack([wo.haar_filter(x[b, h].astype(np.float64), filt[b * H + h].astype(np.float64), L)
                    for b in range(B) for h in range(H)]).reshape(B, H, n, d)
    assert hp.rel_err(y, ref) < 2e-6


def test_rerun_is_bit_identical():
    """Fixed-order reductions: two runs give identical bits (doubles as a race check)."""
    import torch
    cfg = dict(B=2, H=2, n=2048, d=64, L=5, m=128, dtype="bf16", flavour="spikes", seed_base=21, q_mean=0.2)
    p = workloads.make_inputs(**cfg)
    a = hp.gpu_forward_backward(p, cfg)
    b = hp.gpu_forward_backward(p, cfg)
    for k in ("O", "dQ", "dK", "dV", "dWg", "dbg", "domega", "dsigma"):
        assert torch.equal(a[k], b[k]), k


def test_unsupported_shape_raises_without_launch():
    import torch
    from paper_2507_08637_amd import binding
    q = torch.zeros(1, 1, 128, 40, device="cuda")   # head dimension 40: not a multiple of 16
    om = torch.zeros(40, 64, device="cuda")
    one = torch.ones(1, device="cuda")
    with pytest.raises(binding.WersaError) as e:
        binding.wersa_forward(q, q, q, om, one, torch.zeros(1, 4, 40, device="cuda"),
                              torch.zeros(1, 4, device="cuda"), torch.ones(4, device="cuda"), 3)
    assert e.value.status == 2


@pytest.mark.parametrize("path", ["generic_f32", "generic_bf16", "mfma", "mfma256"])
def test_separate_query_and_key_random_matrices(path):
    """WERSA_FLAG_SEPARATE_OMEGA (Algorithm 1's independent W_Q^rand, W_K^rand): omega_rf carries
    two matrices; both paths against the oracle given the same pair."""
    dtype = "f32" if path == "generic_f32" else "bf16"
    cfg = dict(B=2, H=2, n=256, d=64, L=4, m=128, dtype=dtype, flavour="plain", seed_base=3100, q_mean=0.4)
    if path == "mfma256":   # 256 features per pass: the gradient kernels' other loop forms, dV inside the K-side kernel
        cfg.update(m=256)
        path = "mfma"
    p = workloads.make_inputs(**cfg)
    omk = np.random.default_rng(3199).standard_normal(p["Omega"].shape, dtype=np.float32)
    p["OmegaK"] = workloads.round_to_bf16(omk) if dtype == "bf16" else omk
    flags = 2 | (0 if path == "mfma" else 1)
    res = hp.gpu_forward_backward(p, cfg, flags=flags)
    ref = hp.oracle_backward(p, cfg)
    shared = hp.oracle_backward({k: v for k, v in p.items() if k != "OmegaK"}, cfg)
    assert hp.rel_err(res["O"], shared["O"]) > 0.1   # the key-side matrix is really the second one
    if path == "mfma":
        # n = 256, random inputs: plain 1.1e-2 .. 1.6e-2 on dW_g, 2.1e-2 .. 3.2e-2 on d omega
        _check_mfma(res, ref, p, cfg, where="separate omega mfma", noise_limited=True)
    else:
        _check_all(res, ref, TOL[dtype], where=f"separate omega {path}")


@pytest.mark.parametrize("path", ["generic_f32", "generic_bf16", "mfma", "mfma256"])
def test_gate_pooled_over_heads(path):
    """WERSA_FLAG_POOLED_GATE (Algorithm 1's gate: one filter per batch element from the pooled
    queries of all heads) on both paths against the oracle's pooled form."""
    dtype = "f32" if path == "generic_f32" else "bf16"
    cfg = dict(B=2, H=3, n=256, d=64, L=4, m=128, dtype=dtype, flavour="plain", seed_base=3300, q_mean=0.4)
    if path == "mfma256":
        cfg.update(m=256)
        path = "mfma"
    p = workloads.make_inputs(**cfg)
    flags = 4 | (0 if path == "mfma" else 1)
    res = hp.gpu_forward_backward(p, cfg, flags=flags)
    ref = hp.oracle_backward(p, cfg, pooled=True)
    F = res["saved"]["F"].view(cfg["B"], cfg["H"], cfg["L"] + 1)
    assert float((F - F[:, :1]).abs().max().cpu()) == 0.0          # every head of a batch element shares F
    per_head = hp.oracle_backward(p, cfg)
    assert hp.rel_err(res["O"], per_head["O"]) > 1e-2                # and it is not the per-head gate
    if path == "mfma":
        # (un-cancelled scales are the per-head magnitudes: the same order for the pooled sums)
        # (128 features: plain 2.1e-2 on dW_g; 256 features: 7.7e-3)
        _check_mfma(res, ref, p, cfg, where="pooled gate mfma", noise_limited=cfg["m"] == 128, pooled=True)
    else:
        _check_all(res, ref, TOL[dtype], where=f"pooled gate {path}")


@pytest.mark.parametrize("path", ["generic_f32", "generic_bf16", "mfma"])
def test_layernorm_output_stage(path):
    """WERSA_FLAG_LAYERNORM (Algorithm 1's output stage: LayerNorm over the head dimension in
    place of the normaliser) on both paths against the oracle's option; eps = 1e-3 so that the
    eps-order bandwidth gradient is well above rounding."""
    import torch
    from paper_2507_08637_amd import binding
    dtype = "f32" if path == "generic_f32" else "bf16"
    cfg = dict(B=2, H=2, n=320, d=64, L=4, m=128, dtype=dtype, flavour="plain", seed_base=3500, q_mean=0.4)
    p = workloads.make_inputs(**cfg)
    eps = 1e-3
    flags = 8 | (0 if path == "mfma" else 1)
    res = hp.gpu_forward_backward(p, cfg, eps=eps, flags=flags)
    ref = hp.oracle_backward(p, cfg, eps=eps, layernorm=True)
    plain = hp.oracle_backward(p, cfg, eps=eps)
    assert hp.rel_err(res["O"], plain["O"]) > 0.1                    # it is not the Section 3.1 normaliser
    O = res["O"].float()
    assert float(O.mean(dim=-1).abs().max().cpu()) < (1e-5 if dtype == "f32" else 2e-2)
    fwd = hp.oracle_forward(p, cfg, eps=eps, keep=("D",), layernorm=True)
    D = res["saved"]["D"].view(cfg["B"], cfg["H"], cfg["n"])
    assert hp.rel_err(D, fwd["D"]) < TOL[dtype]
    if path == "mfma":
        probe = torch.empty(cfg["B"], cfg["H"], cfg["n"], cfg["d"], dtype=torch.bfloat16, device="cuda")
        assert binding.wersa_path_name(binding.make_desc(probe, cfg["L"], cfg["m"], eps, 1e-6, flags)) == "mfma"
        _check_mfma(res, ref, p, cfg, where="layernorm mfma", eps=eps, layernorm=True)
        assert abs(float(res["dsigma"].cpu()) - ref["dsigma"]) < 5e-2 * abs(ref["dsigma"])
    else:
        _check_all(res, ref, TOL[dtype], where=f"layernorm {path}")
        assert abs(float(res["dsigma"].cpu()) - ref["dsigma"]) < (1e-3 if dtype == "f32" else 2e-2) * abs(ref["dsigma"])


@pytest.mark.parametrize("shape", [dict(B=1, H=2, n=1024, d=64, L=5, m=256, noise=True),    # (plain d omega 2.8e-2)
                                   dict(B=2, H=1, n=832, d=128, L=6, m=256),
                                   dict(B=1, H=2, n=1000, d=64, L=5, m=256, noise=True),    # partial last block (2.2e-2)
                                   dict(B=1, H=2, n=1024, d=64, L=8, m=256)])   # transform deeper than one block
def test_layernorm_output_stage_mfma_shapes(shape):
    """The LayerNorm output stage on the other MFMA kernel variants: 256-feature operand blocks
    (d = 64) and the head dimension 128."""
    import torch
    from paper_2507_08637_amd import binding
    shape = dict(shape)
    noise = shape.pop("noise", False)
    cfg = dict(shape, dtype="bf16", flavour="plain", seed_base=3600, q_mean=0.3)
    p = workloads.make_inputs(**cfg)
    eps = 1e-3
    probe = torch.empty(cfg["B"], cfg["H"], cfg["n"], cfg["d"], dtype=torch.bfloat16, device="cuda")
    assert binding.wersa_path_name(binding.make_desc(probe, cfg["L"], cfg["m"], eps, 1e-6, 8)) == "mfma"
    res = hp.gpu_forward_backward(p, cfg, eps=eps, flags=8)
    ref = hp.oracle_backward(p, cfg, eps=eps, layernorm=True)
    _check_mfma(res, ref, p, cfg, where=f"layernorm mfma {shape}", noise_limited=noise, eps=eps, layernorm=True)
    fwd = hp.oracle_forward(p, cfg, eps=eps, keep=("D",), layernorm=True)
    assert hp.rel_err(res["saved"]["D"].view(cfg["B"], cfg["H"], cfg["n"]), fwd["D"]) < 2e-2
    assert abs(float(res["dsigma"].cpu()) - ref["dsigma"]) < 5e-2 * abs(ref["dsigma"])


@pytest.mark.parametrize("shape", [dict(B=1, H=2, n=1024, d=64, L=8, m=256),      # 16 tiles, blocks of 4 tiles
                                   dict(B=2, H=1, n=4160, d=64, L=12, m=128),     # 65 tiles: one 4096-row block + one tile
                                   dict(B=1, H=1, n=8192, d=64, L=13, m=256, noise=True),     # one block of 128 tiles (one slice, random: plain d omega 3.2e-2)
                                   dict(B=1, H=2, n=640, d=64, L=7, m=128),       # 10 tiles, pairs
                                   dict(B=1, H=2, n=1000, d=64, L=9, m=256),      # partial last tile: 15 tiles + 40 rows
                                   dict(B=1, H=1, n=100, d=64, L=7, m=128, noise=True),       # two tiles, the second partial (6.4e-2)
                                   dict(B=1, H=1, n=2048, d=64, L=8, m=512, noise=True),      # two passes of 256 features (dV inside the K-side kernel) (2.7e-2)
                                   dict(B=1, H=2, n=1024, d=128, L=9, m=128),     # head dimension 128: stage A kernel takes the addends
                                   dict(B=2, H=1, n=4160, d=128, L=12, m=256),
                                   dict(B=1, H=1, n=1000, d=128, L=8, m=128)])    # ... with a partial last tile
def test_deep_transform_on_the_mfma_path(shape):
    """L > 6 stays on the MFMA path: levels up to
    6 inside the kernels, the levels above as per-tile addends built from the tile sums (and,
    backwards, from the tile sums of dX_F, with their share of the band inner products)."""
    import torch
    from paper_2507_08637_amd import binding
    shape = dict(shape)
    noise = shape.pop("noise", False)
    cfg = dict(shape, dtype="bf16", flavour="plain", seed_base=3800, q_mean=0.3)
    probe = torch.empty(cfg["B"], cfg["H"], cfg["n"], cfg["d"], dtype=torch.bfloat16, device="cuda")
    assert binding.wersa_path_name(binding.make_desc(probe, cfg["L"], cfg["m"])) == "mfma"
    p = workloads.make_inputs(**cfg)
    res = hp.gpu_forward_backward(p, cfg)
    ref = hp.oracle_backward(p, cfg)
    _check_mfma(res, ref, p, cfg, where=f"deep mfma {shape}", noise_limited=noise)
    fwd = hp.oracle_forward(p, cfg)
    sl = cfg["B"] * cfg["H"]
    for name in ("qbar", "s", "F", "S", "z", "D"):
        r = fwd[name].reshape((sl,) + fwd[name].shape[2:])
        assert hp.rel_err(res["saved"][name], r) < 2e-2, name


def test_deep_transform_outside_the_mfma_shapes_takes_the_generic_path():
    """L > 6 with a feature count the MFMA path does not take (m % 128 != 0): the default
    selection is the generic path, which meets the bf16 bar."""
    import torch
    from paper_2507_08637_amd import binding
    cfg = dict(B=1, H=2, n=1024, d=128, L=9, m=192, dtype="bf16", flavour="plain", seed_base=3700, q_mean=0.3)
    probe = torch.empty(cfg["B"], cfg["H"], cfg["n"], cfg["d"], dtype=torch.bfloat16, device="cuda")
    assert binding.wersa_path_name(binding.make_desc(probe, cfg["L"], cfg["m"])) == "generic"
    assert binding.wersa_path_name(binding.make_desc(probe, cfg["L"], 128)) == "mfma"
    p = workloads.make_inputs(**cfg)
    res = hp.gpu_forward_backward(p, cfg)
    ref = hp.oracle_backward(p, cfg)
    _check_all(res, ref, TOL["bf16"], where="deep transform, default path")


@pytest.mark.parametrize("shape", [dict(B=2, H=2, n=4096, d=64, L=6, m=256, dtype="bf16"),     # dV inside the K-side kernel
                                   dict(B=1, H=2, n=1000, d=64, L=9, m=256, dtype="bf16"),     # partial last block, deep
                                   dict(B=1, H=2, n=2048, d=128, L=5, m=256, dtype="bf16"),
                                   dict(B=1, H=2, n=1500, d=48, L=4, m=80, dtype="f32")])      # generic path
def test_results_are_bitwise_reproducible(shape):
    """Every reduction runs in a fixed order (no atomics): two runs on the same inputs give the
    same bits in every output, forward and backward."""
    import torch
    cfg = dict(shape, flavour="plain", seed_base=4100, q_mean=0.2)
    p = workloads.make_inputs(**cfg)
    a = hp.gpu_forward_backward(p, cfg)
    b = hp.gpu_forward_backward(p, cfg)
    for name in ("O", "dQ", "dK", "dV", "dWg", "dbg", "domega", "dsigma"):
        assert torch.equal(a[name], b[name]), name
    for name in ("S", "z", "D", "F"):
        assert torch.equal(a["saved"][name], b["saved"][name]), name


@pytest.mark.parametrize("zero", ["K", "V", "Q"])
@pytest.mark.parametrize("shape", [dict(B=1, H=2, n=320, d=64, L=4, m=256, dtype="bf16"),     # MFMA path, dV inside the K-side kernel
                                   dict(B=1, H=2, n=200, d=128, L=5, m=128, dtype="bf16"),    # head dimension 128, partial last block
                                   dict(B=1, H=2, n=200, d=32, L=3, m=48, dtype="f32")])      # generic path
def test_degenerate_all_zero_operand(shape, zero):
    """The degenerate cases of the method.  K = 0: every key feature is ReLU(0) = 0, so S = 0, z = 0,
    D = eps, O = 0 and every gradient is 0 (the ReLU derivative at exactly 0 is 0).  V = 0: O = 0 and
    dQ = dK = 0, dV is not.  Q = 0: the pooled query and every query feature are 0, so O = 0 and
    dK = dV = 0, while dQ = 0 too (derivative at 0).  Everything must come out finite and, where the
    oracle says zero, exactly zero; the rest at the usual tolerance."""
    import torch
    cfg = dict(shape, flavour="plain", seed_base=4300, q_mean=0.2)
    p = workloads.make_inputs(**cfg)
    p[zero] = np.zeros_like(p[zero])
    res = hp.gpu_forward_backward(p, cfg)
    ref = hp.oracle_backward(p, cfg)
    tol = TOL[cfg["dtype"]]
    for name in ("O", "dQ", "dK", "dV", "dWg", "dbg", "domega"):
        got = res[name].float()
        assert bool(torch.isfinite(got).all()), name
        if not np.any(ref[name]):
            assert not bool(got.abs().max() > 0), (name, float(got.abs().max()))
        else:
            assert hp.rel_err(res[name], ref[name]) < tol, (name, hp.rel_err(res[name], ref[name]))
    assert not np.any(ref["O"])      # the premise: the output vanishes in all three cases


@pytest.mark.parametrize("kind", ["mfma", "generic"])
def test_maximum_sequence_length_keeps_convexity_and_periodicity(kind):
    """n = 2^22 (the largest the library takes) on either path, no oracle pass at this size.
    Forward: with V = 1 every output row is (D - eps) / D, a convex combination of ones, so all
    4 M rows must come out as 1, and S must repeat z in every column.  Backward: Q, K and dO repeat
    a block of 4096 random rows; every per-row result (O, dQ, dK, dV) depends on its 64-row block
    and on slice-wide sums only, so it must repeat with the same period, bit for bit.  Row-index
    arithmetic that wraps or skips anywhere in the 4 M rows breaks one of the two."""
    import torch
    from paper_2507_08637_amd import binding
    n, L, P = 1 << 22, 6, 4096
    d, m, dt = (64, 256, torch.bfloat16) if kind == "mfma" else (16, 32, torch.float32)
    g = torch.Generator(device="cuda")
    g.manual_seed(4200)
    rnd = lambda *sh: torch.randn(*sh, device="cuda", generator=g, dtype=torch.float32)
    tile = lambda base: base.to(dt).repeat(n // P, 1).view(1, 1, n, d).contiguous()
    Q, K, dO = tile(rnd(P, d)), tile(rnd(P, d)), tile(rnd(P, d))
    V = torch.ones(1, 1, n, d, device="cuda", dtype=dt)
    Om = rnd(d, m).to(dt)
    sigma = torch.ones(1, device="cuda")
    Wg, bg, om = 0.1 * rnd(1, L + 1, d), 0.1 * rnd(1, L + 1), torch.ones(L + 1, device="cuda")
    desc = binding.make_desc(Q, L, m)
    assert binding.wersa_path_name(desc) == kind
    out, saved = binding.wersa_forward(Q, K, V, Om, sigma, Wg, bg, om, L)
    sv = binding.saved_views(desc, saved)
    o = out.float()
    assert torch.isfinite(o).all()
    assert (o - 1.0).abs().max().item() < (1e-2 if kind == "mfma" else 1e-4)   # rounding of (D - eps) / D
    assert (sv["D"] > 0).all()
    S, z = sv["S"].reshape(m, d), sv["z"].reshape(m)
    assert torch.allclose(S, z[:, None].expand(m, d), rtol=1e-4, atol=0.0)
    gr = binding.wersa_backward(Q, K, V, Om, sigma, Wg, bg, om, out, dO, saved, L)
    torch.cuda.synchronize()
    for name in ("dq", "dk", "dv", "dgate_w", "dgate_b", "dscale_w", "dsigma"):
        assert torch.isfinite(gr[name].float()).all(), name
    periodic = lambda x: bool((x.view(n // P, P, d) == x.view(n // P, P, d)[0]).all())
    assert periodic(sv["D"].reshape(n, 1).expand(n, d)), "D"
    for name, x in (("O", out), ("dQ", gr["dq"]), ("dK", gr["dk"]), ("dV", gr["dv"])):
        assert periodic(x), name
    assert gr["dv"].float().abs().max().item() > 0


# ------------------------------------------------------------------ benchmark configurations
def test_config1_tiny_fp32():
    cfg, p = workloads.make_config(1, backward=True)
    res = hp.gpu_forward_backward(p, cfg)
    ref = hp.oracle_backward(p, cfg)
    _check_all(res, ref, 1e-4, where="config1")


def test_config2_bf16_forward():
    cfg, p = workloads.make_config(2)
    res = hp.gpu_forward_backward(p, cfg, backward=False)
    ref = hp.oracle_forward(p, cfg, keep=("O",))
    assert hp.rel_err(res["O"], ref["O"]) < 2e-2


# Bounds on the per-block and per-element error figures at full size (helpers.err_stats), next to the
# 2e-2 Frobenius bar.  O and dV are smooth functions of the inputs: every 64-row block and every
# element must sit near the bf16 output rounding (2^-9).  dQ and dK contain the ReLU derivative, a
# binary decision: where a pre-activation is within fp16 rounding of zero the kernel and float64
# decide differently and that row's gradient moves by one feature's whole contribution, so single
# rows and the blocks that hold them carry errors well above the tensor's average (measured: worst
# block 4e-2 .. 6e-2, largest element error 4e-2 .. 1.1e-1 of the largest element); the bounds
# below leave a factor of two over that and still reject a wholly wrong block (relative error 1)
# or a wrong element of the size of the largest.
BLOCK_BOUNDS = dict(O=dict(worst_block=1e-2, maxabs=1e-2), dV=dict(worst_block=1e-2, maxabs=1e-2),
                    dQ=dict(worst_block=0.15, maxabs=0.25), dK=dict(worst_block=0.15, maxabs=0.25))


def _check_blocks(res, ref, where):
    for name, bounds in BLOCK_BOUNDS.items():
        st = hp.err_stats(res[name], ref[name])
        print(where, name, {k: f"{v:.2e}" for k, v in st.items()}, flush=True)
        for k, limit in bounds.items():
            assert st[k] < limit, (where, name, k, st[k])


def _full_size_check(idx):
    """Full-size GPU run against the oracle on EVERY (batch, head) slice: the plain 2e-2 on O, dQ,
    dK, dV and on the gate-parameter gradients, which sum over all slices, plus the per-block and
    per-element bounds above."""
    cfg, p = workloads.make_config(idx)
    res = hp.gpu_forward_backward(p, cfg)
    ref = hp.oracle_backward(p, cfg)
    _check_all(res, ref, 2e-2, where=f"config{idx}")
    _check_blocks(res, ref, f"config{idx}")
    for b in range(cfg["B"]):
        for h in range(cfg["H"]):
            for name in ("O", "dQ", "dK", "dV"):
                e = hp.rel_err(res[name][b, h], ref[name][b, h])
                assert e < 2e-2, (name, b, h, e)


def test_config3_spikes_forward_backward():
    _full_size_check(3)


def test_config4_long_sequence_forward_backward():
    _full_size_check(4)
