"""Parity of the attention block (projections around the core) through the C-ABI against the
float64 oracle.  Storage is bf16: the oracle takes the same bf16-rounded inputs in float64 and
rounds the stored intermediates (Q', K', V', A and their gradients) to bf16 where the kernel
stores them, so that each stage is compared on the same numbers; tolerance 2e-2 relative
Frobenius error per output, 2e-3 for a single projection (one bf16 rounding of a float32 sum).
"""
import numpy as np
import pytest

from paper_2507_08637_amd import workloads
from tests import helpers as hp

pytestmark = pytest.mark.gpu

BLOCK_SHAPES = [
    dict(B=1, H=4, n=256, d=64, L=4, m=128),     # hidden 256: one tile in each direction
    dict(B=2, H=4, n=384, d=128, L=6, m=256, noise=True),    # hidden 512, 768 tokens: 3 x 2 tiles, head dim 128 (plain d omega 2.1e-2)
    dict(B=3, H=8, n=256, d=64, L=3, m=128),     # hidden 512, weight-gradient split over tokens
]


def _gpu_block(p, cfg, backward=True):
    import torch
    from paper_2507_08637_amd import binding
    dev = "cuda:0"
    bf = lambda a: torch.from_numpy(a).to(dev).to(torch.bfloat16)
    f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)
    t = {k: bf(p[k]) for k in ("X", "WQ", "WK", "WV", "WO", "Omega")}
    t.update({k: f32(p[k]) for k in ("Wg", "bg", "omega")})
    t["sigma"] = torch.tensor([float(p["sigma"])], dtype=torch.float32, device=dev)
    H, L = cfg["H"], cfg["L"]
    y, saved = binding.wersa_block_forward(t["X"], t["WQ"], t["WK"], t["WV"], t["WO"], H, t["Omega"], t["sigma"],
                                           t["Wg"], t["bg"], t["omega"], L)
    desc = binding.make_block_desc(t["X"], H, L, cfg["m"])
    res = dict(Y=y)
    res.update({k: v.clone() for k, v in binding.block_saved_views(desc, saved).items() if k != "core"})
    if backward:
        g = binding.wersa_block_backward(t["X"], t["WQ"], t["WK"], t["WV"], t["WO"], H, t["Omega"], t["sigma"],
                                         t["Wg"], t["bg"], t["omega"], bf(p["dY"]), saved, L)
        res.update(dX=g["dx"], dWQ=g["dwq"], dWK=g["dwk"], dWV=g["dwv"], dWO=g["dwo"], dWg=g["dgate_w"],
                   dbg=g["dgate_b"], domega=g["dscale_w"], dsigma=g["dsigma"])
    torch.cuda.synchronize()
    return res


def _oracle_block(p, cfg, proj_dtype=None):
    from oracle import wersa_oracle as wo
    return wo.block_backward(p["X"], p["WQ"], p["WK"], p["WV"], p["WO"], cfg["H"], p["Omega"], float(p["sigma"]),
                             p["Wg"], p["bg"], p["omega"], cfg["L"], p["dY"], proj_dtype=proj_dtype,
                             store=lambda a: workloads.round_to_bf16(a).astype(np.float64))


@pytest.mark.parametrize("shape", BLOCK_SHAPES, ids=lambda s: "B{B}H{H}n{n}d{d}L{L}m{m}".format(**s))
def test_block_forward_backward(shape):
    from oracle import wersa_oracle as wo
    cfg = dict(shape)
    noise = cfg.pop("noise", False)
    p = workloads.make_block_inputs(**cfg, seed_base=9100, x_mean=0.0)
    res = _gpu_block(p, cfg)
    ref = _oracle_block(p, cfg)
    proj = {k: hp.rel_err(res[k], ref[k]) for k in ("Qp", "Kp", "Vp")}
    print(shape, "projections", {k: f"{v:.2e}" for k, v in proj.items()}, flush=True)
    assert all(v < 2e-3 for v in proj.values()), proj
    ref16 = _oracle_block(p, cfg, proj_dtype=np.float16)
    errs = {k: hp.rel_err(res[k], ref[k]) for k in ("A", "Y", "dX", "dWQ", "dWK", "dWV", "dWO")}
    errs16 = {k: hp.rel_err(res[k], ref16[k]) for k in ("A", "Y", "dX", "dWQ", "dWK", "dWV", "dWO")}
    print(shape, {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    print(shape, "fp16 decision", {k: f"{v:.2e}" for k, v in errs16.items()}, flush=True)
    bad = {k: v for k, v in errs.items() if not v < 2e-2}
    assert not bad, bad
    # Gate-parameter gradients: cancelling sums on random inputs, bounded against their
    # un-cancelled magnitude on the core problem the block hands to the core (as in the core's
    # MFMA parity tests), with the ReLU decision taken on fp16-rounded X_F on both sides.
    H = cfg["H"]
    core_p = dict(Q=wo.split_heads(ref["Qp"], H), K=wo.split_heads(ref["Kp"], H), V=wo.split_heads(ref["Vp"], H),
                  dO=wo.split_heads(ref["dA"], H), Omega=p["Omega"], Wg=p["Wg"], bg=p["bg"], omega=p["omega"],
                  sigma=p["sigma"])
    plain = {k: hp.rel_err(res[k], ref[k]) for k in ("dWg", "dbg", "domega")}
    print(shape, "gate grads, plain relative", {k: f"{v:.2e}" for k, v in plain.items()}, flush=True)
    if not noise:   # the plain bar, except where the sums sit at their noise floor on these small random inputs
        assert all(v < 2e-2 for v in plain.values()), plain
        return
    scales = hp.gate_grad_scales(core_p, dict(cfg, d=cfg["d"]))
    gerr = {k: hp.scaled_err(res[k], ref16[k], scales[k]) for k in ("dWg", "dbg", "domega")}
    print(shape, "gate grads vs un-cancelled scale", {k: f"{v:.2e}" for k, v in gerr.items()}, flush=True)
    assert all(v < 5e-2 for v in gerr.values()), gerr


@pytest.mark.parametrize("case", ["large", "tiny"])
def test_block_input_range(case):
    """The block hands the core the largest |Q'| per 128 rows and 64 columns from the epilogue of
    its W^Q product, so the fp16 operands of the projection (Section 3.1 step 7) carry the same
    per-slice power-of-two scale as in the core's own entry points: token features of the order
    2^13 (the filtered rows would overflow fp16 without the scale) or 2^-16 (they would sit among
    its subnormals; the bandwidth stays above the descriptor's floor), with the bandwidth scaled alike, must meet the bar of order-one inputs.
    The factor is a power of two f, so the whole computation is homogeneous: against the run on the
    unscaled inputs, Y and the weight gradients carry f, dX carries 1, d b_g and d omega carry f and
    d W_g (logits kept where they were by W_g / f) carries f^2 - to the last bits, which also holds
    the gate-parameter gradients (noise-limited against the oracle at this size) to account."""
    import torch
    cfg = dict(B=1, H=4, n=256, d=64, L=4, m=128)
    p0 = workloads.make_block_inputs(**cfg, seed_base=9400, x_mean=0.0)
    f = 2.0 ** 13 if case == "large" else 2.0 ** -16
    p = dict(p0)
    p["X"] = workloads.round_to_bf16(p0["X"] * np.float32(f))     # a power of two: still exact bf16 values
    p["sigma"] = np.float32(float(p0["sigma"]) * f)
    p["Wg"] = (p0["Wg"] / np.float32(f)).astype(np.float32)        # keeps the gate logits where they were
    res = _gpu_block(p, cfg)
    ref = _oracle_block(p, cfg)
    errs = {k: hp.rel_err(res[k], ref[k]) for k in ("A", "Y", "dX", "dWQ", "dWK", "dWV", "dWO")}
    print("block input range", case, {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    assert all(bool(torch.isfinite(res[k].float()).all()) for k in ("Y", "dX", "dWQ", "dWg"))
    assert all(v < 2e-2 for v in errs.values()), errs
    base = _gpu_block(p0, cfg)
    power = dict(Y=1, A=1, dX=0, dWQ=1, dWK=1, dWV=1, dWO=1, dWg=2, dbg=1, domega=1)
    hom = {k: hp.rel_err(res[k].double() / f ** e, base[k].double().cpu().numpy()) for k, e in power.items()}
    print("block input range", case, "against the unscaled run", {k: f"{v:.1e}" for k, v in hom.items()}, flush=True)
    assert all(v < 1e-6 for v in hom.values()), hom


def test_block_results_are_bitwise_reproducible():
    """The split-k partials of the weight gradients are summed in a fixed order and the core has
    no atomics: two runs of the block on the same inputs give the same bits."""
    import torch
    cfg = dict(B=2, H=4, n=384, d=128, L=6, m=256)
    p = workloads.make_block_inputs(**cfg, seed_base=9300, x_mean=0.1)
    a = _gpu_block(p, cfg)
    b = _gpu_block(p, cfg)
    for name in ("Y", "A", "dX", "dWQ", "dWK", "dWV", "dWO", "dWg", "dbg", "domega", "dsigma"):
        assert torch.equal(a[name], b[name]), name


def test_block_gradient_of_query_weights_with_shifted_input():
    """With a non-zero token mean of X the weight gradient dW^Q = X^T dQ' picks up the rank-one
    term (sum_t X_t) (dqbar / n)^T: the pooled-query gradient, a cancelling sum whose error is
    bounded only against its un-cancelled magnitude (see the gate gradients).  The part of dW^Q
    orthogonal to the mean row of X does not see it and must meet the plain tolerance, as must
    every other output."""
    cfg = dict(B=2, H=4, n=256, d=64, L=4, m=128)
    p = workloads.make_block_inputs(**cfg, seed_base=9200, x_mean=0.3)
    res = _gpu_block(p, cfg)
    ref16 = _oracle_block(p, cfg, proj_dtype=np.float16)
    errs = {k: hp.rel_err(res[k], ref16[k]) for k in ("A", "Y", "dX", "dWK", "dWV", "dWO")}
    print("shifted X", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    assert all(v < 2e-2 for v in errs.values()), errs
    xbar = p["X"].astype(np.float64).reshape(-1, p["X"].shape[2]).mean(axis=0)
    u = xbar / np.linalg.norm(xbar)
    gpu = res["dWQ"].double().cpu().numpy()
    proj_gpu = gpu - np.outer(u, u @ gpu)
    proj_ref = ref16["dWQ"] - np.outer(u, u @ ref16["dWQ"])
    e = float(np.linalg.norm(proj_gpu - proj_ref) / np.linalg.norm(proj_ref))
    print(f"shifted X: dWQ orthogonal to the mean row {e:.2e}, whole {hp.rel_err(res['dWQ'], ref16['dWQ']):.2e}",
          flush=True)
    assert e < 2e-2


def test_config5_block_full_size():
    """Configuration 5 at full size (B=2, H=16, n=65536, d=128, hidden 2048) through the block
    entry points against the oracle's block on the whole problem: every projection, every head's
    A, dA, dQ', dK', dV', the outputs Y and dX on every token, the four weight gradients and the
    gate-parameter gradients (which sum over all 32 slices), plus per-block and per-element bounds
    on the per-head tensors (see BLOCK_BOUNDS in the core's parity tests)."""
    import time
    import torch
    from paper_2507_08637_amd import binding
    from tests.test_gpu_parity import BLOCK_BOUNDS
    cfg = dict(workloads.CONFIGS[5])
    B, H, n, d, L, m = (cfg[k] for k in ("B", "H", "n", "d", "L", "m"))
    hidden = H * d
    p = workloads.make_block_inputs(B, H, n, d, L, m, seed_base=5000)
    dev = "cuda:0"
    bf = lambda a: torch.from_numpy(a).to(dev).to(torch.bfloat16)
    f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)
    t = {k: bf(p[k]) for k in ("X", "WQ", "WK", "WV", "WO", "Omega", "dY")}
    t.update({k: f32(p[k]) for k in ("Wg", "bg", "omega")})
    t["sigma"] = torch.tensor([float(p["sigma"])], dtype=torch.float32, device=dev)
    desc = binding.make_block_desc(t["X"], H, L, m)
    assert binding.wersa_path_name(binding.WersaDesc(B, H, n, d, L, m, 1, 1e-6, 1e-6, n * hidden, d, hidden, 0)) == "mfma"
    y, saved = binding.wersa_block_forward(t["X"], t["WQ"], t["WK"], t["WV"], t["WO"], H, t["Omega"], t["sigma"],
                                           t["Wg"], t["bg"], t["omega"], L)
    wsb = torch.empty(binding.load_library().wersa_block_workspace_bytes(desc, 1), dtype=torch.uint8, device=dev)
    g = binding.wersa_block_backward(t["X"], t["WQ"], t["WK"], t["WV"], t["WO"], H, t["Omega"], t["sigma"],
                                     t["Wg"], t["bg"], t["omega"], t["dY"], saved, L, workspace=wsb)
    torch.cuda.synchronize()
    sv = binding.block_saved_views(desc, saved)
    wv = binding.block_workspace_views(desc, wsb)
    print("config5 block: GPU forward and backward done", flush=True)
    # the oracle, one batch element at a time (they are independent; gradients of parameters and
    # weights sum over them), so that each call finishes in about a minute and prints when it has
    t0 = time.time()
    ref = None
    per_token = ("Y", "A", "Qp", "Kp", "Vp", "dA", "dQp", "dKp", "dVp", "dX")
    for b in range(B):
        rb = _oracle_block(dict(p, X=p["X"][b:b + 1], dY=p["dY"][b:b + 1]), cfg)
        print(f"config5 block: oracle, batch element {b} done after {time.time() - t0:.0f} s", flush=True)
        if ref is None:
            ref = rb
        else:
            for k in rb:
                ref[k] = np.concatenate([ref[k], rb[k]], axis=0) if k in per_token else ref[k] + rb[k]
        del rb

    def check(name, gpu, r, tol=2e-2):
        e = hp.rel_err(gpu, r)
        print(f"config5 block {name}: {e:.2e}", flush=True)
        assert e < tol, (name, e)

    for name in ("Qp", "Kp", "Vp"):
        check(name, sv[name], ref[name], tol=2e-3)
    check("dA", wv["dA"], ref["dA"], tol=2e-3)
    check("A", sv["A"], ref["A"])
    for name in ("dQp", "dKp", "dVp"):
        check(name, wv[name], ref[name])
    check("Y", y, ref["Y"])
    check("dX", g["dx"], ref["dX"])
    for name, key in (("dWQ", "dwq"), ("dWK", "dwk"), ("dWV", "dwv"), ("dWO", "dwo")):
        check(name, g[key], ref[name])
    for name, key in (("dWg", "dgate_w"), ("dbg", "dgate_b"), ("domega", "dscale_w")):
        check(name, g[key], ref[name])
    # per head: Frobenius error of every (batch, head) slice, worst 64-row block, largest element error
    from oracle import wersa_oracle as wo
    for name, gpu, bound in (("A", sv["A"], "O"), ("dQp", wv["dQp"], "dQ"), ("dKp", wv["dKp"], "dK"),
                             ("dVp", wv["dVp"], "dV")):
        gh = gpu.view(B, n, H, d).permute(0, 2, 1, 3)
        rh = wo.split_heads(ref[name], H)
        st = hp.err_stats(gh, rh)
        print(f"config5 block {name} per-head figures", {k: f"{v:.2e}" for k, v in st.items()}, flush=True)
        for k, limit in BLOCK_BOUNDS[bound].items():
            assert st[k] < limit, (name, k, st[k])
        for b in range(B):
            for h in range(H):
                e = hp.rel_err(gh[b, h], rh[b, h])
                assert e < 2e-2, (name, b, h, e)


def test_block_rejects_unsupported_shapes():
    import torch
    from paper_2507_08637_amd import binding
    x = torch.zeros(1, 256, 192, dtype=torch.bfloat16, device="cuda")   # hidden 192: not a multiple of 256
    desc = binding.make_block_desc(x, 3, 2, 128)
    assert binding.load_library().wersa_block_saved_bytes(desc) == 0
    x = torch.zeros(1, 192, 256, dtype=torch.bfloat16, device="cuda")   # 192 tokens
    desc = binding.make_block_desc(x, 4, 2, 128)
    assert binding.load_library().wersa_block_workspace_bytes(desc, 1) == 0
