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
    dict(B=2, H=4, n=384, d=128, L=6, m=256),    # hidden 512, 768 tokens: 3 x 2 tiles, head dim 128
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
    scales = hp.gate_grad_scales(core_p, dict(cfg, d=cfg["d"]))
    gerr = {k: hp.scaled_err(res[k], ref16[k], scales[k]) for k in ("dWg", "dbg", "domega")}
    print(shape, "gate grads vs un-cancelled scale", {k: f"{v:.2e}" for k, v in gerr.items()}, flush=True)
    assert all(v < 5e-2 for v in gerr.values()), gerr


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
    entry points.  The oracle recomputes head h of both batches from the inputs alone (its own
    projections, core forward and backward), which pins: the projections, A, dA, dQ', dK', dV' on
    those slices and the column (row) blocks of the four weight gradients that belong to head h
    (they sum over both batches).  Y and dX mix all heads of a token; they are checked as the
    stated product of the kernel's own stage inputs on sampled tokens (a property of the stage
    that holds at any size), the stage inputs themselves being pinned per slice as above."""
    import torch
    from oracle import wersa_oracle as wo
    from paper_2507_08637_amd import binding
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

    h = 11
    cols = slice(h * d, (h + 1) * d)
    rb = lambda a: workloads.round_to_bf16(a).astype(np.float64)
    f64 = lambda a: np.asarray(a, np.float64)
    WQ, WK, WV, WO = (f64(p[k]) for k in ("WQ", "WK", "WV", "WO"))
    Om, Wg_h, bg_h, om = f64(p["Omega"]), f64(p["Wg"][h]), f64(p["bg"][h]), f64(p["omega"])
    sigma = float(p["sigma"])
    dW = {k: np.zeros((hidden, d)) for k in ("dWQ", "dWK", "dWV")}
    dWO_rows = np.zeros((d, hidden))

    def gpu_np(tensor):
        return tensor.double().cpu().numpy()

    def check(name, gpu, ref, tol=2e-2):
        e = float(np.linalg.norm(gpu - ref) / np.linalg.norm(ref))
        print(f"config5 block {name}: {e:.2e}", flush=True)
        assert e < tol, (name, e)

    for b in range(B):
        Xb, dYb = f64(p["X"][b]), f64(p["dY"][b])
        Qs, Ks, Vs = rb(Xb @ WQ[:, cols]), rb(Xb @ WK[:, cols]), rb(Xb @ WV[:, cols])
        for name, ref in (("Qp", Qs), ("Kp", Ks), ("Vp", Vs)):
            check(f"b{b} h{h} {name}", gpu_np(sv[name][b][:, cols]), ref, tol=2e-3)
        fw = wo.forward_slice(Qs, Ks, Vs, Om, sigma, Wg_h, bg_h, om, L, 1e-6, 1e-6)
        As = rb(fw["O"])
        check(f"b{b} h{h} A", gpu_np(sv["A"][b][:, cols]), As)
        dAs = rb(dYb @ WO[cols, :].T)
        check(f"b{b} h{h} dA", gpu_np(wv["dA"][b][:, cols]), dAs, tol=2e-3)
        bw = wo.backward_slice(Qs, Ks, Vs, Om, sigma, Wg_h, bg_h, om, L, 1e-6, 1e-6, dAs, fwd=fw)
        for name, key in (("dQp", "dQ"), ("dKp", "dK"), ("dVp", "dV")):
            ref = rb(bw[key])
            check(f"b{b} h{h} {name}", gpu_np(wv[name][b][:, cols]), ref)
            dW["dW" + name[1].upper()] += Xb.T @ ref
        dWO_rows += As.T @ dYb
        del Xb, dYb, fw, bw
    for name, key in (("dWQ", "dwq"), ("dWK", "dwk"), ("dWV", "dwv")):
        check(f"{name}[:, head {h}]", gpu_np(g[key][:, cols]), dW[name])
    check(f"dWO[head {h}, :]", gpu_np(g["dwo"][cols, :]), dWO_rows)

    # Y = A W^out and dX = dQ' W^Q^T + dK' W^K^T + dV' W^V^T on sampled tokens, from the kernel's
    # own stage inputs.
    r = np.random.default_rng(55)
    toks = [(int(r.integers(B)), int(r.integers(n))) for _ in range(48)] + [(0, 0), (B - 1, n - 1)]
    bi = torch.tensor([b for b, _ in toks], device=dev)
    ti = torch.tensor([tt for _, tt in toks], device=dev)
    rows = lambda tensor: gpu_np(tensor[bi, ti])
    check("Y on sampled tokens", rows(y), rows(sv["A"]) @ WO, tol=5e-3)
    check("dX on sampled tokens", rows(g["dx"]),
          rows(wv["dQp"]) @ WQ.T + rows(wv["dKp"]) @ WK.T + rows(wv["dVp"]) @ WV.T, tol=5e-3)


def test_block_rejects_unsupported_shapes():
    import torch
    from paper_2507_08637_amd import binding
    x = torch.zeros(1, 256, 192, dtype=torch.bfloat16, device="cuda")   # hidden 192: not a multiple of 256
    desc = binding.make_block_desc(x, 3, 2, 128)
    assert binding.load_library().wersa_block_saved_bytes(desc) == 0
    x = torch.zeros(1, 192, 256, dtype=torch.bfloat16, device="cuda")   # 192 tokens
    desc = binding.make_block_desc(x, 4, 2, 128)
    assert binding.load_library().wersa_block_workspace_bytes(desc, 1) == 0
