"""The autograd wrappers (same kernels, reached through loss.backward()) and replay of the whole
forward+backward inside a captured HIP graph."""
import numpy as np
import pytest

from paper_2507_08637_amd import workloads
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def test_autograd_matches_oracle():
    import torch
    from paper_2507_08637_amd.autograd import wersa_attention
    cfg = dict(B=1, H=2, n=256, d=64, L=4, m=128, dtype="bf16", flavour="plain", seed_base=77, q_mean=0.5)
    p = workloads.make_inputs(**cfg)
    t = hp.to_device(p, "bf16")
    leaves = {k: t[k].clone().requires_grad_(True) for k in ("Q", "K", "V", "Wg", "bg", "omega", "sigma")}
    out = wersa_attention(leaves["Q"], leaves["K"], leaves["V"], t["Omega"], leaves["sigma"], leaves["Wg"],
                          leaves["bg"], leaves["omega"], cfg["L"])
    (out.float() * t["dO"].float()).sum().backward()
    torch.cuda.synchronize()
    ref = hp.oracle_backward(p, cfg)
    assert hp.rel_err(out, ref["O"]) < 2e-2
    for name, key in (("Q", "dQ"), ("K", "dK"), ("V", "dV")):
        assert hp.rel_err(leaves[name].grad, ref[key]) < 2e-2, name
    for name in ("Wg", "bg", "omega", "sigma"):
        assert leaves[name].grad is not None and torch.isfinite(leaves[name].grad).all()


def test_forward_backward_replays_in_a_captured_graph():
    """Capture one forward+backward on a side stream into a HIP graph, replay it three times with
    eager work and synchronisation in between, and require every replay to reproduce the eager
    result bit for bit (the library enqueues kernels only: no allocation, no memset, no host sync)."""
    import torch
    from paper_2507_08637_amd import binding
    cfg = dict(B=2, H=2, n=512, d=64, L=5, m=256, dtype="bf16", flavour="plain", seed_base=91, q_mean=0.3)
    p = workloads.make_inputs(**cfg)
    t = hp.to_device(p, "bf16")
    L = cfg["L"]
    desc = binding.make_desc(t["Q"], L, cfg["m"])
    saved, ws_f = binding.alloc_like(desc, t["Q"], 0)
    _, ws_b = binding.alloc_like(desc, t["Q"], 1)
    out = torch.empty_like(t["Q"])
    grads = None

    def step():
        nonlocal grads
        binding.wersa_forward(t["Q"], t["K"], t["V"], t["Omega"], t["sigma"], t["Wg"], t["bg"], t["omega"], L,
                              out=out, saved=saved, workspace=ws_f)
        grads = binding.wersa_backward(t["Q"], t["K"], t["V"], t["Omega"], t["sigma"], t["Wg"], t["bg"],
                                       t["omega"], out, t["dO"], saved, L, workspace=ws_b, grads=grads)

    step()
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in grads.items()}
    eager["out"] = out.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        out.zero_()
        for v in grads.values():
            v.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager["out"]), rep
        for k, v in grads.items():
            assert torch.equal(v, eager[k]), (rep, k)
